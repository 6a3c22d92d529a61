"""GPU parity, one case per compiled form of the store and gather kernels.

The quantize-append and dequant-gather kernels are templates over the input / output type,
the lanes per quant-group, the summary source, the code width, the metadata kind and the
number of token rows a lane keeps in flight; the host picks the form from the configuration
and the launch size.  The tests in test_gpu_parity.py sample those forms through realistic
shapes; the cases here walk through every combination with small tiles, so that no compiled
form goes to a user without having been compared with the oracle (codes, scale / zero and
dequantized values bit-exact, summary keys within one float32 ulp)."""
import itertools

import pytest
import torch

from tests import harness as H

pytestmark = pytest.mark.gpu

TDT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}
D = 128          # every quant-group width divides it; 16 token rows per pass of a workgroup


@pytest.fixture(scope="module")
def oqm():
    from paper_2510_18269_amd import oqm as m      # raises if the library is not built
    assert torch.cuda.is_available()
    return m


def _run(oqm, *, qaxis, dt, gs, sep, bits, meta, G, frames, heads, seed):
    st, mem = H.make_pair(oqm, n_layers=1, n_kv_heads=heads, n_q_heads=2 * heads, head_dim=D, group_tokens=G,
                          qgroup=gs, capacity=frames, in_dtype=dt, qaxis=qaxis, bits=bits, meta=meta)
    try:
        g = torch.Generator().manual_seed(seed)
        shape = (frames, 1, heads, G, D)
        k = (torch.randn(shape, generator=g) * 1.5).to(TDT[dt])
        v = torch.randn(shape, generator=g).to(TDT[dt])
        ks = torch.randn(shape, generator=g).to(TDT[dt]) if sep else None
        H.append_both(oqm, st, mem, k, v, ks)
        H.compare_storage(st, mem)
        q = torch.randn(1, 2 * heads, 2, D, generator=g).to(TDT[dt])
        r = H.full_path_check(oqm, st, mem, q, min(3, frames))
        assert r["k_eff"] == min(3, frames)
    finally:
        mem.close()


# head_dim axis: input type x lanes per quant-group x summary source x code width x metadata kind
# x launch form (at most 768 tiles: 1024 threads per tile, four rows of a lane in flight; more:
# 256 threads, two rows per trip, V tiles cut into chunks).  The group size cycles through 16 / 100 / 180 tokens = 1 / 7 / 12 row
# passes: the gather's two forms (whole tile up to four passes, else chunks of at most three).
_HD = list(itertools.product(("bf16", "f16", "f32"), (8, 16, 32, 64, 128), (False, True), (4, 2),
                             ("f32", "bf16")))


@pytest.mark.parametrize("dt", ("bf16", "f16", "f32"))
def test_every_form_of_the_head_dim_axis_kernels(oqm, dt):
    n = 0
    for i, (dti, gs, sep, bits, meta) in enumerate(_HD):
        if dti != dt:
            continue
        G = (16, 100, 180)[i % 3]
        _run(oqm, qaxis=0, dt=dt, gs=gs, sep=sep, bits=bits, meta=meta, G=G, frames=3, heads=2, seed=5000 + i)
        # 195 frames x 2 heads x (K, V) = 780 tiles: the streaming form of the same kernel
        # (40 token rows: a V tile is two chunks of 20)
        _run(oqm, qaxis=0, dt=dt, gs=gs, sep=sep, bits=bits, meta=meta, G=40, frames=195, heads=2, seed=6000 + i)
        n += 2
    assert n == 80


# token axis: input type x summary source x rows kept in registers (4 / 8 / 13 / none, picked from
# the row passes per tile: 1, 7, 12, 15) x code width x metadata kind
_TOK = list(itertools.product(("bf16", "f16", "f32"), (False, True), (16, 100, 180, 230), (4, 2),
                              ("f32", "bf16")))


@pytest.mark.parametrize("dt", ("bf16", "f16", "f32"))
def test_every_form_of_the_token_axis_kernels(oqm, dt):
    n = 0
    for i, (dti, sep, G, bits, meta) in enumerate(_TOK):
        if dti != dt:
            continue
        _run(oqm, qaxis=1, dt=dt, gs=64, sep=sep, bits=bits, meta=meta, G=G, frames=3, heads=2, seed=7000 + i)
        n += 1
    assert n == 32
