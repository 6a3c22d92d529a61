"""The retrieval entry point that allocates nothing (`tom_oqm_retrieve_noalloc`: the score step's
scratch is a fixed device array inside the library) against `tom_oqm_retrieve` with a
caller-given workspace, through the C ABI.  Same kernels, so every output must be identical
bit for bit: scores, indices, active K and V.  Two calls in a row, the second on a smaller
input, so that what the first call left in the shared array would show if anything read it."""
import numpy as np
import pytest
import torch

import synth_kv
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oqm():
    from paper_2510_18269_amd import oqm as m      # raises if the library is not built
    assert torch.cuda.is_available()
    return m


def _both_ways(oqm, mem, w, q, n_layers, t_q, k, path, prefix, sys_k, sys_v):
    """One retrieval through each entry point on the same inputs; returns the two output sets."""
    L, Hk, d, G = n_layers, w.n_kv_heads, w.head_dim, w.group_tokens
    T = mem.n_groups
    tdt = mem.out_torch_dtype()
    outs = []
    for noalloc in (False, True):
        rows = prefix + k * G
        ko = torch.zeros((L, Hk, rows, d), dtype=tdt, device="cuda")
        vo = torch.zeros((L, Hk, rows, d), dtype=tdt, device="cuda")
        ko.view(torch.int16).fill_(0x7FC1)
        vo.view(torch.int16).fill_(0x7FC1)
        scores = torch.full((L, T + 5), float("nan"), dtype=torch.float32, device="cuda")
        idx = torch.full((L, k), -7, dtype=torch.int32, device="cuda")
        qd = q[:L, :, :t_q].contiguous().cuda()
        sk = sys_k[:L].contiguous().cuda() if prefix else None
        sv = sys_v[:L].contiguous().cuda() if prefix else None
        if noalloc:
            k_eff = oqm.tom_oqm_retrieve_noalloc(mem.handle, 0, L, qd, t_q, k, scores, T + 5, idx, ko, vo,
                                                 path=path, prefix_rows=prefix, sys_k=sk, sys_v=sv)
        else:
            ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, t_q, path, False),
                             dtype=torch.uint8, device="cuda")
            k_eff = oqm.tom_oqm_retrieve(mem.handle, 0, L, qd, t_q, k, scores, T + 5, idx, ko, vo, ws,
                                         path=path, prefix_rows=prefix, sys_k=sk, sys_v=sv)
        torch.cuda.synchronize()
        outs.append((k_eff, scores.cpu().numpy().view(np.uint32), idx.cpu().numpy(), H.bits(ko), H.bits(vo)))
    return outs


@pytest.mark.parametrize("path_name", ["mean_query", "token_gemm"])
def test_retrieve_noalloc_matches_retrieve_on_two_calls_in_a_row(oqm, path_name):
    path = oqm.TOM_SCORE_MEAN_QUERY if path_name == "mean_query" else oqm.TOM_SCORE_TOKEN_GEMM
    w = synth_kv.Workload("X", 3, 4, 28, 128, 50, 70, 64, 24, 7, "bf16", "cosine", 4242, "layer_std", 35)
    st, mem = H.pair_for(oqm, w)
    try:
        for f in (0, 35):
            kk, vv = synth_kv.kv_frames(w, f, 35)
            H.append_both(oqm, st, mem, kk, vv)
        q = synth_kv.query(w)
        g = torch.Generator().manual_seed(9)
        tdt = mem.out_torch_dtype()
        sys_k = torch.randn(w.n_layers, w.n_kv_heads, 3, w.head_dim, generator=g).to(tdt)
        sys_v = torch.randn(w.n_layers, w.n_kv_heads, 3, w.head_dim, generator=g).to(tdt)
        # first call: all layers, the whole query, with a system prefix; second call: fewer
        # layers, fewer query tokens, fewer groups asked for, no prefix
        for (nl, tq, k, prefix) in ((3, 24, 7, 3), (2, 5, 4, 0)):
            a, b = _both_ways(oqm, mem, w, q, nl, tq, k, path, prefix, sys_k, sys_v)
            assert a[0] == b[0] == k
            assert np.array_equal(a[1], b[1]), "scores differ between the two entry points"
            assert np.array_equal(a[2], b[2]), "indices differ between the two entry points"
            assert np.array_equal(a[3], b[3]) and np.array_equal(a[4], b[4]), "active K/V differ"
            # and the result is the oracle's (the bar of the other parity tests)
            ref_scores = H.orc.score_groups(st, H.bits(q[:nl, :, :tq].contiguous()), H.DT["bf16"][0], n_layers=nl)
            ref_idx, k_eff = H.orc.topk(ref_scores, k)
            assert np.array_equal(b[2], ref_idx)
            sc = b[1].view(np.float32)[:, :w.n_frames].astype(np.float64)
            assert np.all(np.abs(sc - ref_scores) <= H.score_bound(st, q, ref_scores))
    finally:
        mem.close()


def test_retrieve_noalloc_refuses_what_its_scratch_cannot_hold(oqm):
    w = synth_kv.Workload("X", 2, 4, 28, 128, 9, 4, 64, 8, 2, "bf16", "cosine", 77, "layer_std", 4)
    st, mem = H.pair_for(oqm, w)
    try:
        kk, vv = synth_kv.kv_frames(w, 0, 4)
        H.append_both(oqm, st, mem, kk, vv)
        t_q = 2048                                        # 2 x 2048 x 512 doubles = 16 MiB > 8 MiB
        assert oqm.tom_oqm_score_workspace_bytes(mem.handle, 2, t_q, oqm.TOM_SCORE_TOKEN_GEMM, False) \
            > oqm.tom_oqm_static_scratch_bytes() == 8 << 20
        q = torch.zeros((2, 28, t_q, 128), dtype=torch.bfloat16, device="cuda")
        scores = torch.zeros((2, 4), dtype=torch.float32, device="cuda")
        idx = torch.zeros((2, 2), dtype=torch.int32, device="cuda")
        ko = torch.zeros((2, 4, 18, 128), dtype=torch.bfloat16, device="cuda")
        vo = torch.zeros_like(ko)
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_retrieve_noalloc(mem.handle, 0, 2, q, t_q, 2, scores, 4, idx, ko, vo,
                                         path=oqm.TOM_SCORE_TOKEN_GEMM)
        assert e.value.status == oqm.TOM_ERR_UNSUPPORTED and "static scratch" in str(e.value)
        torch.cuda.synchronize()
        assert int(idx.abs().sum()) == 0 and float(scores.abs().sum()) == 0.0      # nothing was queued
    finally:
        mem.close()
