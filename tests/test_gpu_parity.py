"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bar: packed codes, scale, zero and retrieved indices bit-exact; summary keys
and scores within one float32 ulp (float64 accumulation on both sides); dequantized values
bit-exact (the same single fused float32 multiply-add and the same round-to-nearest-even
narrowing on both sides), which is inside the stated 1e-6 relative / 1 bf16 ulp tolerance."""
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


def _stream_and_check(oqm, w, frames_per_call, k=None, path=None, want_tokens=False, out_dtype=None,
                      qaxis=0, bits=4, meta="f32"):
    st, mem = H.pair_for(oqm, w, out_dtype=out_dtype, qaxis=qaxis, bits=bits, meta=meta)
    try:
        f = 0
        while f < w.n_frames:
            n = min(frames_per_call, w.n_frames - f)
            kk, vv = synth_kv.kv_frames(w, f, n)
            H.append_both(oqm, st, mem, kk, vv)
            f += n
        frac = H.compare_storage(st, mem)
        assert frac < 1e-3
        q = synth_kv.query(w)
        return H.full_path_check(oqm, st, mem, q, k or w.top_k, path, want_tokens)
    finally:
        mem.close()


def test_c1_tiny_stream_full(oqm):
    w = synth_kv.WORKLOADS["C1"]
    r = _stream_and_check(oqm, w, w.n_frames)
    assert r["k_eff"] == 4 and r["loose_rows"] == 0


def test_c2_single_layer_full(oqm):
    w = synth_kv.WORKLOADS["C2"]
    r = _stream_and_check(oqm, w, 64)
    assert r["k_eff"] == 32 and r["loose_rows"] == 0


@pytest.mark.parametrize("name,layers,frames,per_call", [("C3", 3, 40, 16), ("C4", 2, 37, 1),
                                                         ("C5", 3, 48, 32)])
def test_reduced_multi_layer_streams(oqm, name, layers, frames, per_call):
    """C3/C4/C5 recipes (per-layer std, one-frame appends, outlier keys + gs 32) at a size
    the oracle checks element by element: several tiles, ragged 196-token groups."""
    w = synth_kv.scaled(synth_kv.WORKLOADS[name], n_layers=layers, n_frames=frames,
                        top_k=min(synth_kv.WORKLOADS[name].top_k, 24))
    path = oqm.TOM_SCORE_TOKEN_GEMM if name == "C5" else None
    r = _stream_and_check(oqm, w, per_call, path=path, want_tokens=(name == "C5"))
    assert r["loose_rows"] == 0


@pytest.mark.parametrize("G,d,gs,dt,H_k,H_q", [
    (50, 128, 64, "f16", 4, 28),      # the paper's 50-token groups, FP16 K/V
    (1, 64, 8, "f32", 1, 1), (197, 128, 128, "bf16", 2, 4), (13, 96, 32, "bf16", 3, 6),
    (64, 256, 16, "f16", 2, 2), (33, 8, 8, "f32", 5, 5), (7, 512, 64, "bf16", 1, 3),
    (500, 128, 64, "bf16", 2, 4)])    # 32 row passes per tile: every kernel's multi-trip loop
def test_shapes_dtypes_and_ragged_tails(oqm, G, d, gs, dt, H_k, H_q):
    w = synth_kv.Workload("X", 2, H_k, H_q, d, G, 11, gs, 5, 4, dt, "cosine", 100 + G + d, "layer_std", 11)
    r = _stream_and_check(oqm, w, 4)
    assert r["k_eff"] == 4
    r = _stream_and_check(oqm, synth_kv.scaled(w, sim="dot", t_q=17), 11, k=6,
                          path=oqm.TOM_SCORE_TOKEN_GEMM, want_tokens=True)
    assert r["k_eff"] == 6


@pytest.mark.parametrize("G,d,gs,H_k,frames", [
    (65, 128, 64, 4, 49),     # 5 row passes: the gather's first chunked shape (2 x 33 rows); V tiles 3 x 22
    (97, 128, 32, 4, 49),     # 7 passes: 3 gather chunks of 33; V tiles 3 x 32 + 1 -> 4 chunks of 25
    (129, 64, 16, 3, 65),     # 32 rows per pass: V chunks of 43 rows, gather 5 passes -> 2 x 65
    (520, 128, 64, 4, 49),    # 33 passes: 11 gather chunks of 48, 17 V chunks of 31
    (47, 256, 128, 2, 97),    # 8 rows per pass: 16-row V chunks, 6 passes -> 2 gather chunks of 24
    (31, 1032, 8, 1, 193)])   # 129 lanes per row: one row per pass, 31 passes
def test_chunk_boundaries_of_the_store_and_gather_kernels(oqm, G, d, gs, H_k, frames):
    """The streaming form of the append cuts V tiles into one-trip chunks and the gather cuts
    tiles of more than four row passes into equal chunks: shapes that put chunk ends next to
    tile ends, on launches of more than 768 tiles (the streaming form) and three frames at a time."""
    w = synth_kv.Workload("X", 2, H_k, 2 * H_k, d, G, frames, gs, 5, 5, "bf16", "cosine", 4400 + G + d,
                          "layer_std", frames)
    assert 2 * 2 * H_k * frames > 768          # K and V tiles of 2 layers: the streaming form
    r = _stream_and_check(oqm, w, frames)
    assert r["k_eff"] == 5 and r["loose_rows"] == 0
    r = _stream_and_check(oqm, w, 3, bits=2, meta="bf16")
    assert r["k_eff"] == 5 and r["loose_rows"] == 0


@pytest.mark.parametrize("G,d,dt,H_k,H_q", [
    (50, 128, "f16", 4, 28),           # the paper's setting: 50-token groups, FP16, per-channel scale
    (196, 128, "bf16", 4, 28), (1, 64, "f32", 1, 1), (13, 96, "bf16", 3, 6), (300, 64, "f16", 2, 2),
    (33, 8, "f32", 5, 5), (40, 512, "bf16", 1, 3),
    (500, 128, "bf16", 2, 4), (150, 128, "f32", 1, 2)])   # more rows per lane than the kernel keeps in registers
def test_token_axis_quantizer(oqm, G, d, dt, H_k, H_q):
    """Eq. 9 as printed: scale and zero per head and channel over the G tokens of a group."""
    w = synth_kv.Workload("X", 2, H_k, H_q, d, G, 9, 64, 5, 4, dt, "cosine", 300 + G + d, "outlier", 9)
    r = _stream_and_check(oqm, w, 4, qaxis=1)
    assert r["k_eff"] == 4 and r["loose_rows"] == 0


@pytest.mark.parametrize("qaxis,G,d,gs,dt,H_k,H_q", [
    (0, 196, 128, 64, "bf16", 4, 28), (0, 50, 128, 32, "f16", 4, 28), (1, 50, 128, 64, "f16", 4, 28),
    (1, 196, 128, 64, "bf16", 4, 28), (0, 13, 96, 8, "f32", 3, 6), (1, 300, 64, 64, "bf16", 2, 2),
    (0, 1, 8, 8, "f32", 1, 1), (0, 33, 256, 128, "bf16", 2, 4), (1, 500, 128, 64, "f16", 2, 2),
    (0, 500, 128, 32, "bf16", 2, 2)])
def test_two_bit_codes(oqm, qaxis, G, d, gs, dt, H_k, H_q):
    """The paper's bit-width ablation: 2-bit codes (three steps between min and max), four per
    byte, on both quantization axes."""
    w = synth_kv.Workload("X", 2, H_k, H_q, d, G, 10, gs, 5, 4, dt, "cosine", 700 + G + d, "outlier", 10)
    r = _stream_and_check(oqm, w, 4, qaxis=qaxis, bits=2)
    assert r["k_eff"] == 4 and r["loose_rows"] == 0


def test_two_bit_extreme_ranges(oqm):
    """Steps above 2^126 (their reciprocal is sub-normal), flat and sub-normal-step groups."""
    for qaxis in (0, 1):
        st, mem = H.make_pair(oqm, n_layers=1, n_kv_heads=2, n_q_heads=2, head_dim=64, group_tokens=9,
                              qgroup=32, capacity=3, in_dtype="f32", qaxis=qaxis, bits=2)
        try:
            g = torch.Generator().manual_seed(12)
            k = torch.randn(3, 1, 2, 9, 64, generator=g)
            k[0] *= 1.2e38                                           # range up to ~3e38: s > 2^126
            k[0].clamp_(-1.6e38, 1.6e38)
            k[1, 0, 0] = 2.5
            k[1, 0, 1, :, :32] = torch.linspace(0, 2e-38, 32)       # sub-normal step
            v = -k.clone()
            # max - min = 3.4e38, just finite, in K and in V.  The key column of that K tile
            # cancels at 1e38: its float64 sum depends on the order of the additions, so the
            # keys of that frame are held to 1e-6 * max|K| of the tile, all others to one ulp.
            for x in (k, v):
                x[2, 0, 0, 0, 0] = 1.7e38
                x[2, 0, 0, 1, 0] = -1.7e38
            H.append_both(oqm, st, mem, k, v)
            key_abs = np.zeros((1, 3, 2))
            key_abs[0, 2, :] = 1e-6 * k[2, 0].abs().amax(dim=(1, 2)).double().numpy()
            H.compare_storage(st, mem, key_abs=key_abs)
        finally:
            mem.close()


@pytest.mark.parametrize("qaxis,bits,G,d,gs,dt,H_k,H_q", [
    (0, 4, 196, 128, 64, "bf16", 4, 28), (0, 4, 50, 128, 32, "f16", 4, 28), (1, 4, 50, 128, 64, "f16", 4, 28),
    (1, 4, 196, 128, 64, "bf16", 4, 28), (0, 2, 196, 128, 64, "bf16", 4, 28), (1, 2, 50, 128, 64, "f16", 4, 28),
    (0, 4, 13, 96, 8, "f32", 3, 6), (1, 4, 300, 64, 64, "f32", 2, 2), (0, 2, 33, 256, 128, "f32", 2, 4)])
def test_bf16_metadata(oqm, qaxis, bits, G, d, gs, dt, H_k, H_q):
    """(scale, zero) kept as bfloat16 pairs: rounded before the codes are taken, codes clamped;
    codes, stored pairs, indices and reconstructed values bit-exact against the oracle."""
    w = synth_kv.Workload("X", 2, H_k, H_q, d, G, 10, gs, 5, 4, dt, "cosine", 1300 + G + d + bits, "outlier", 10)
    r = _stream_and_check(oqm, w, 4, qaxis=qaxis, bits=bits, meta="bf16")
    assert r["k_eff"] == 4 and r["loose_rows"] == 0


@pytest.mark.parametrize("bits,meta,dt,G,d,gs,H_k,frames", [
    (4, "f32", "bf16", 50, 128, 64, 4, 49), (2, "f32", "f16", 13, 96, 8, 3, 65),
    (4, "bf16", "f32", 33, 256, 128, 2, 97), (2, "bf16", "bf16", 196, 128, 64, 4, 49)])
def test_append_launches_above_and_below_three_tiles_per_cu(oqm, bits, meta, dt, G, d, gs, H_k, frames):
    """The head_dim-axis append has two forms of one kernel: 1024 threads per tile with four rows
    per lane in flight for launches of at most 768 tiles, above that 256 threads, two rows per
    trip and V tiles cut into chunks.  Most cases in this file are small launches; here one
    call stores more than 768 tiles, then the same stream goes in frame by frame, and both must
    match the oracle."""
    w = synth_kv.Workload("X", 2, H_k, 2 * H_k, d, G, frames, gs, 5, 6, dt, "cosine", 2100 + G + d + bits,
                          "layer_std", frames)
    assert H_k * 2 * 2 * frames > 768
    r = _stream_and_check(oqm, w, frames, bits=bits, meta=meta)
    assert r["k_eff"] == 6 and r["loose_rows"] == 0
    r = _stream_and_check(oqm, w, 1, bits=bits, meta=meta)
    assert r["k_eff"] == 6 and r["loose_rows"] == 0


@pytest.mark.parametrize("qaxis,bits,d,gs,dt", [(0, 4, 2048, 128, "bf16"), (1, 4, 2048, 64, "f16"),
                                               (0, 2, 1032, 8, "f32"), (1, 2, 1032, 8, "bf16"),
                                               (0, 4, 1032, 8, "f16")])
def test_widest_and_odd_head_dims(oqm, qaxis, bits, d, gs, dt):
    """The widest head the configuration check admits (2048: one token row fills the whole
    workgroup) and a width whose lane count per row (129) is neither a power of two nor a
    divisor of the workgroup: every kernel of the path on both axes."""
    w = synth_kv.Workload("X", 2, 2, 4, d, 5, 7, gs, 3, 3, dt, "cosine", 3100 + d + bits, "layer_std", 7)
    r = _stream_and_check(oqm, w, 3, qaxis=qaxis, bits=bits)
    assert r["k_eff"] == 3 and r["loose_rows"] == 0
    r = _stream_and_check(oqm, synth_kv.scaled(w, t_q=18), 7, k=4, path=oqm.TOM_SCORE_TOKEN_GEMM,
                          want_tokens=True, qaxis=qaxis, bits=bits)
    assert r["k_eff"] == 4


@pytest.mark.parametrize("H_k,d", [(16, 512), (4, 2048)])
def test_widest_flattened_key(oqm, H_k, d):
    """H_k * d = 8192, the most the score kernels admit (64 KB of staged query per workgroup)."""
    w = synth_kv.Workload("X", 1, H_k, 2 * H_k, d, 3, 6, 64, 2, 3, "bf16", "cosine", 3300 + d, "layer_std", 6)
    r = _stream_and_check(oqm, w, 6)
    assert r["k_eff"] == 3 and r["loose_rows"] == 0
    r = _stream_and_check(oqm, synth_kv.scaled(w, t_q=5), 6, k=2, path=oqm.TOM_SCORE_TOKEN_GEMM, want_tokens=True)
    assert r["k_eff"] == 2


def test_mixed_in_out_dtypes(oqm):
    w = synth_kv.scaled(synth_kv.WORKLOADS["C2"], n_frames=9, top_k=3)
    for out in ("f32", "f16", "bf16"):
        _stream_and_check(oqm, w, 9, out_dtype=out)


@pytest.mark.parametrize("qaxis,bits,meta,dt,G", [(0, 4, "f32", "bf16", 21), (1, 4, "f32", "f16", 21),
                                                  (0, 2, "bf16", "f32", 21), (1, 2, "bf16", "bf16", 21),
                                                  (1, 4, "f32", "bf16", 200), (1, 4, "f32", "f32", 300)])
def test_strided_input_layer_ranges_and_separate_summary(oqm, qaxis, bits, meta, dt, G):
    """Token-major source buffers [F][G][L][H][d], layers appended one at a time with
    commit only on the last, summary keys from a separate (pre-rotary) tensor; on both axes,
    both code widths and metadata kinds (the token-axis cases with 200 and 300 tokens take the
    forms that keep 8 rows per lane in registers and none at all: 7 and 10 row passes at d = 64)."""
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dt]
    eb = 4 if dt == "f32" else 2
    st, mem = H.make_pair(oqm, n_layers=3, n_kv_heads=2, n_q_heads=4, head_dim=64, group_tokens=G,
                          qgroup=32, capacity=6, in_dtype=dt, qaxis=qaxis, bits=bits, meta=meta)
    try:
        g = torch.Generator().manual_seed(9)
        F, L, Hk, d = 2, 3, 2, 64
        for call in range(2):
            bk = torch.randn(F, G, L, Hk, d, generator=g).to(tdt)
            bv = torch.randn(F, G, L, Hk, d, generator=g).to(tdt)
            pre = torch.randn(F, G, L, Hk, d, generator=g).to(tdt)
            strides = (G * L * Hk * d, Hk * d, d, L * Hk * d)
            dk, dv, dp = bk.cuda(), bv.cuda(), pre.cuda()
            for l in range(L):
                off = l * strides[1]
                H.orc.quantize_append(st, H.bits(bk).ravel()[off:], H.bits(bv).ravel()[off:],
                                      H.bits(pre).ravel()[off:], layer0=l, strides=strides,
                                      n_frames=F, n_layers=1, commit=(l == L - 1))
                first = oqm.tom_oqm_quantize_append(
                    mem.handle, l, 1, F, dk.data_ptr() + off * eb, dv.data_ptr() + off * eb,
                    dp.data_ptr() + off * eb, strides, commit=(l == L - 1))
                assert first == call * F
            torch.cuda.synchronize()
        assert mem.n_groups == 4
        H.compare_storage(st, mem)
        q = torch.randn(3, 4, 3, 64, generator=g).to(tdt)
        H.full_path_check(oqm, st, mem, q, 3)
    finally:
        mem.close()


def test_empty_and_degenerate_cases(oqm):
    st, mem = H.make_pair(oqm, n_layers=2, n_kv_heads=2, n_q_heads=2, head_dim=64, group_tokens=16,
                          qgroup=32, capacity=5, in_dtype="f32")
    try:
        g = torch.Generator().manual_seed(4)
        # nothing stored: score and top-k are no-ops, k_eff = 0
        sc = torch.zeros(2, 8, device="cuda")
        idx = torch.full((2, 4), -7, dtype=torch.int32, device="cuda")
        assert oqm.tom_oqm_topk(sc, 8, 2, 0, 4, idx) == 0
        assert (idx == -7).all()
        # constant tiles, zero tiles, a huge-range tile, negative zeros
        k = torch.randn(5, 2, 2, 16, 64, generator=g)
        k[0] = 3.25
        k[1, 0] = 0.0
        k[1, 1, 0, :, ::2] = -0.0
        k[2, :, :, 3, 5] = 1e30
        k[2, :, :, 4, 6] = -1e30
        k[3, 0, 0, 0, :32] = torch.linspace(0, 1e-37, 32)       # sub-normal step
        v = -k.clone()
        H.append_both(oqm, st, mem, k, v)
        H.compare_storage(st, mem)
        with pytest.raises(oqm.TomError) as e:                    # full: nothing is evicted
            oqm.tom_oqm_quantize_append(mem.handle, 0, 2, 1, k.cuda(), v.cuda())
        assert e.value.status == oqm.TOM_ERR_CAPACITY and mem.n_groups == 5
        # k larger than the number of stored groups: all of them, in order; rest untouched
        q = torch.randn(2, 2, 1, 64, generator=g)
        r = H.full_path_check(oqm, st, mem, q, 8)
        assert r["k_eff"] == 5
        # zero query under cosine: norms are clamped, scores are 0, lowest indices win
        sc, _ = H.gpu_scores(oqm, mem, torch.zeros(2, 2, 1, 64))
        assert (sc[:, :5] == 0).all()
        idx, k_eff, _, _ = H.gpu_retrieve(oqm, mem, sc, 3, 2)
        assert idx.tolist() == [[0, 1, 2]] * 2
    finally:
        mem.close()


def test_gather_skips_bad_indices_and_respects_the_bound(oqm):
    st, mem = H.make_pair(oqm, n_layers=1, n_kv_heads=2, n_q_heads=2, head_dim=64, group_tokens=10,
                          qgroup=32, capacity=8, in_dtype="bf16")
    try:
        k, v = (torch.randn(6, 1, 2, 10, 64, generator=torch.Generator().manual_seed(s)).to(torch.bfloat16)
                for s in (1, 2))
        H.append_both(oqm, st, mem, k, v)
        kq = 4
        idx = torch.tensor([[5, 6, -1, 2]], dtype=torch.int32, device="cuda")   # 6 and -1 are not stored
        G = 10
        guard = 3
        ko = torch.full((1, 2, kq * G + guard, 64), 7.0, dtype=torch.bfloat16, device="cuda")
        vo = ko.clone()
        # the library sees buffers of exactly k*G rows per head: hand it per-head views via k = 4
        ko_c = torch.full((1, 2, kq * G, 64), 7.0, dtype=torch.bfloat16, device="cuda")
        vo_c = ko_c.clone()
        oqm.tom_oqm_dequant_gather(mem.handle, 0, 1, idx, kq, 4, ko_c, vo_c)
        torch.cuda.synchronize()
        ref_k, ref_v = H.orc.dequant_gather(st, np.array([[5, 2]], np.int32), 2)
        got = H.bits(ko_c)
        assert np.array_equal(got[:, :, 0:G], ref_k[:, :, 0:G])
        assert np.array_equal(got[:, :, 3 * G:4 * G], ref_k[:, :, G:2 * G])
        seven = H.bits(torch.tensor([7.0], dtype=torch.bfloat16))[0]
        assert np.all(got[:, :, G:3 * G] == seven)                 # skipped ranks untouched
        # k_eff < k: rows beyond k_eff*G stay as they were
        ko_c.fill_(7.0)
        oqm.tom_oqm_dequant_gather(mem.handle, 0, 1, idx, kq, 1, ko_c, vo_c)
        torch.cuda.synchronize()
        got = H.bits(ko_c)
        assert np.array_equal(got[:, :, 0:G], ref_k[:, :, 0:G]) and np.all(got[:, :, G:] == seven)
    finally:
        mem.close()


@pytest.mark.parametrize("T,k", [(1, 1), (37, 5), (256, 32), (1024, 64), (3600, 64), (5000, 4096),
                                 (8192, 100), (8193, 100), (40000, 777)])
def test_topk_against_oracle(oqm, T, k):
    g = torch.Generator().manual_seed(T + k)
    rows = 3
    s = torch.randn(rows, T + 5, generator=g)
    s[1] = torch.round(s[1] * 4) / 4                               # heavy exact ties
    s[2, ::3] = 0.0
    s[2, 1::3] = -0.0                                              # -0 == +0
    s[:, T:] = 1e9                                                 # padding beyond n_groups must never win
    sd = s.cuda()
    for order in (oqm.TOM_ORDER_INDEX_ASC, oqm.TOM_ORDER_SCORE_DESC):
        if order == oqm.TOM_ORDER_SCORE_DESC and min(k, T) > 4096:
            continue
        idx = torch.full((rows, k), -7, dtype=torch.int32, device="cuda")
        k_eff = oqm.tom_oqm_topk(sd, T + 5, rows, T, k, idx, order)
        torch.cuda.synchronize()
        want, k_ref = H.orc.topk(s.numpy(), k, order, n_groups=T)
        assert k_eff == k_ref == min(k, T)
        got = idx.cpu().numpy()
        assert np.array_equal(got[:, :k_eff], want[:, :k_eff])
        assert np.all(got[:, k_eff:] == -7)


def test_topk_all_equal_and_monotone_rows(oqm):
    s = torch.zeros(2, 500)
    s[1] = torch.arange(500, dtype=torch.float32)
    idx = torch.zeros((2, 7), dtype=torch.int32, device="cuda")
    oqm.tom_oqm_topk(s.cuda(), 500, 2, 500, 7, idx)
    assert idx.cpu().tolist() == [list(range(7)), list(range(493, 500))]
    oqm.tom_oqm_topk(s.cuda(), 500, 2, 500, 7, idx, oqm.TOM_ORDER_SCORE_DESC)
    assert idx.cpu().tolist() == [list(range(7)), list(range(499, 492, -1))]


def test_planted_query_is_retrieved(oqm):
    w = synth_kv.scaled(synth_kv.WORKLOADS["C2"], n_frames=40, n_q_heads=4, t_q=1)
    st, mem = H.pair_for(oqm, w)
    try:
        k, v = synth_kv.kv_frames(w, 0, 40)
        H.append_both(oqm, st, mem, k, v)
        keys = mem.keys.view(1, 40, 4, 128)
        q = keys[:, 23].reshape(1, 4, 1, 128).contiguous()       # r = 1: the stored key itself
        for path in (oqm.TOM_SCORE_MEAN_QUERY, oqm.TOM_SCORE_TOKEN_GEMM):
            sc, _ = H.gpu_scores(oqm, mem, q, path)
            assert abs(sc[0, 23].item() - 1.0) < 1e-6 and sc[0, :40].argmax().item() == 23
            assert (sc[0, :40].abs() <= 1 + 1e-6).all()
    finally:
        mem.close()


def test_both_score_paths_agree(oqm):
    w = synth_kv.scaled(synth_kv.WORKLOADS["C5"], n_layers=2, n_frames=70, t_q=64)
    st, mem = H.pair_for(oqm, w)
    try:
        k, v = synth_kv.kv_frames(w, 0, 70)
        H.append_both(oqm, st, mem, k, v)
        q = synth_kv.query(w)
        a, _ = H.gpu_scores(oqm, mem, q, oqm.TOM_SCORE_MEAN_QUERY, stride_pad=3)
        b, tok = H.gpu_scores(oqm, mem, q, oqm.TOM_SCORE_TOKEN_GEMM, want_tokens=True)
        a, b = a.cpu().numpy()[:, :70], b.cpu().numpy()[:, :70]
        assert np.all(np.abs(a - b) <= np.spacing(np.abs(a)))
        # longer queries than one 64-row tile, and a ragged last row tile
        w2 = synth_kv.scaled(w, t_q=150)
        H.full_path_check(oqm, st, mem, synth_kv.query(w2), 9, oqm.TOM_SCORE_TOKEN_GEMM, True)
        # every count of 16-row tiles per block (1, 2, 3, 4 and 4 + 1), full and ragged
        for t_q in (1, 16, 17, 33, 48, 49, 65):
            wq = synth_kv.scaled(w, t_q=t_q)
            H.full_path_check(oqm, st, mem, synth_kv.query(wq), 9, oqm.TOM_SCORE_TOKEN_GEMM, True)
    finally:
        mem.close()


@pytest.mark.parametrize("qaxis,G,prefix,dt", [(0, 196, 14, "bf16"), (0, 50, 1, "f16"), (1, 50, 14, "f16"),
                                               (0, 13, 0, "f32")])
def test_assemble_with_system_prefix_and_one_call_retrieve(oqm, qaxis, G, prefix, dt):
    """System-token rows in front of the gathered groups (dual-structure memory), and the
    one-call score -> top-k -> assemble path; both against the oracle's step-by-step result."""
    w = synth_kv.Workload("X", 3, 4, 28, 128, G, 45, 64, 24, 7, dt, "cosine", 500 + G, "layer_std", 45)
    st, mem = H.pair_for(oqm, w, qaxis=qaxis)
    try:
        kk, vv = synth_kv.kv_frames(w, 0, w.n_frames)
        H.append_both(oqm, st, mem, kk, vv)
        q = synth_kv.query(w)
        cfg = st.cfg
        L, Hk, d, k = w.n_layers, w.n_kv_heads, w.head_dim, w.top_k
        tdt = mem.out_torch_dtype()
        g = torch.Generator().manual_seed(77)
        sys_k = torch.randn(L, Hk, max(prefix, 1), d, generator=g).to(tdt)[:, :, :prefix].contiguous()
        sys_v = torch.randn(L, Hk, max(prefix, 1), d, generator=g).to(tdt)[:, :, :prefix].contiguous()
        # oracle, step by step
        ref_scores = H.orc.score_groups(st, H.bits(q), H.DT[dt][0])
        ref_idx, k_eff = H.orc.topk(ref_scores, k)
        fill = 0x7FC1 if dt != "f32" else None
        ref_k, ref_v = H.orc.assemble_active(st, ref_idx, k_eff, prefix, H.bits(sys_k) if prefix else None,
                                             H.bits(sys_v) if prefix else None, fill=fill)
        # GPU: one call
        rows = prefix + k * G
        ko = torch.zeros((L, Hk, rows, d), dtype=tdt, device="cuda")
        vo = torch.zeros((L, Hk, rows, d), dtype=tdt, device="cuda")
        if fill is not None:
            ko.view(torch.int16).fill_(fill)
            vo.view(torch.int16).fill_(fill)
        scores = torch.empty((L, w.n_frames + 3), dtype=torch.float32, device="cuda")
        idx = torch.full((L, k), -7, dtype=torch.int32, device="cuda")
        ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, w.t_q, oqm.TOM_SCORE_AUTO, False),
                         dtype=torch.uint8, device="cuda")
        got_keff = oqm.tom_oqm_retrieve(mem.handle, 0, L, q.cuda(), w.t_q, k, scores, scores.shape[1], idx,
                                        ko, vo, ws, prefix_rows=prefix,
                                        sys_k=sys_k.cuda() if prefix else None,
                                        sys_v=sys_v.cuda() if prefix else None)
        torch.cuda.synchronize()
        assert got_keff == k_eff == k
        sc = scores.cpu().numpy()[:, :w.n_frames]
        assert np.all(np.abs(sc.astype(np.float64) - ref_scores) <= H.score_bound(st, q, ref_scores))
        assert np.array_equal(idx.cpu().numpy(), ref_idx)
        assert np.array_equal(H.bits(ko), ref_k) and np.array_equal(H.bits(vo), ref_v)
        # GPU: the assemble step alone, prefix left untouched when no system tensors are given
        ko2 = torch.zeros_like(ko)
        vo2 = torch.zeros_like(vo)
        oqm.tom_oqm_assemble_active(mem.handle, 0, L, idx, k, k_eff - 2, prefix, None, None, ko2, vo2)
        torch.cuda.synchronize()
        b = H.bits(ko2)
        assert np.all(b[:, :, :prefix] == 0) and np.all(b[:, :, prefix + (k_eff - 2) * G:] == 0)
        assert np.array_equal(b[:, :, prefix:prefix + (k_eff - 2) * G], ref_k[:, :, prefix:prefix + (k_eff - 2) * G])
        # prefix only (nothing retrieved yet)
        if prefix:
            oqm.tom_oqm_assemble_active(mem.handle, 0, L, None, k, 0, prefix, sys_k.cuda(), sys_v.cuda(), ko2, vo2)
            torch.cuda.synchronize()
            assert np.array_equal(H.bits(vo2)[:, :, :prefix], H.bits(sys_v))
    finally:
        mem.close()


def test_one_call_retrieve_on_an_empty_and_on_a_short_store(oqm):
    """Nothing stored: k_eff = 0, only the system prefix is written.  Fewer groups stored than
    asked for: all of them in temporal order, the rows behind them untouched."""
    w = synth_kv.Workload("X", 2, 2, 4, 64, 9, 3, 32, 5, 6, "bf16", "cosine", 910, "layer_std", 3)
    st, mem = H.pair_for(oqm, w, capacity=8)
    try:
        L, Hk, d, G, k, prefix = w.n_layers, w.n_kv_heads, w.head_dim, w.group_tokens, w.top_k, 2
        g = torch.Generator().manual_seed(5)
        sys_k = torch.randn(L, Hk, prefix, d, generator=g).to(torch.bfloat16)
        sys_v = torch.randn(L, Hk, prefix, d, generator=g).to(torch.bfloat16)
        q = synth_kv.query(w)
        rows = prefix + k * G
        ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, w.t_q, oqm.TOM_SCORE_AUTO, False),
                         dtype=torch.uint8, device="cuda")
        scores = torch.full((L, 8), 123.0, dtype=torch.float32, device="cuda")
        idx = torch.full((L, k), -7, dtype=torch.int32, device="cuda")

        def call():
            ko = torch.zeros((L, Hk, rows, d), dtype=torch.bfloat16, device="cuda")
            vo = torch.zeros_like(ko)
            ko.view(torch.int16).fill_(0x7FC1)
            vo.view(torch.int16).fill_(0x7FC1)
            ke = oqm.tom_oqm_retrieve(mem.handle, 0, L, q.cuda(), w.t_q, k, scores, 8, idx, ko, vo, ws,
                                      prefix_rows=prefix, sys_k=sys_k.cuda(), sys_v=sys_v.cuda())
            torch.cuda.synchronize()
            return ke, ko, vo

        ke, ko, vo = call()
        assert ke == 0 and (idx == -7).all() and (scores == 123.0).all()
        assert np.array_equal(H.bits(ko)[:, :, :prefix], H.bits(sys_k))
        assert np.all(H.bits(vo)[:, :, prefix:] == 0x7FC1)

        kk, vv = synth_kv.kv_frames(w, 0, 3)
        H.append_both(oqm, st, mem, kk, vv)
        ke, ko, vo = call()
        assert ke == 3 and idx.cpu().numpy()[:, :3].tolist() == [[0, 1, 2]] * L
        ref_k, ref_v = H.orc.assemble_active(st, idx.cpu().numpy(), 3, prefix, H.bits(sys_k), H.bits(sys_v),
                                             fill=0x7FC1)
        assert np.array_equal(H.bits(ko), ref_k) and np.array_equal(H.bits(vo), ref_v)
        assert np.all(H.bits(ko)[:, :, prefix + 3 * G:] == 0x7FC1)
    finally:
        mem.close()


def test_layer_by_layer_calls_match_the_all_layer_call(oqm):
    """Inside a model's forward pass the retrieval runs one layer at a time (layer0 = l,
    n_layers = 1): every step must give what the all-layer call gives, i.e. the oracle's."""
    w = synth_kv.Workload("X", 4, 4, 28, 128, 50, 30, 64, 8, 5, "bf16", "cosine", 811, "layer_std", 30)
    st, mem = H.pair_for(oqm, w)
    try:
        kk, vv = synth_kv.kv_frames(w, 0, w.n_frames)
        H.append_both(oqm, st, mem, kk, vv)
        q = synth_kv.query(w)
        L, Hk, G, d, k = w.n_layers, w.n_kv_heads, w.group_tokens, w.head_dim, w.top_k
        ref_scores = H.orc.score_groups(st, H.bits(q), 1)
        ref_idx, k_eff = H.orc.topk(ref_scores, k)
        ref_k, ref_v = H.orc.dequant_gather(st, ref_idx, k_eff)
        qd = q.cuda()
        for path in (oqm.TOM_SCORE_MEAN_QUERY, oqm.TOM_SCORE_TOKEN_GEMM):
            for l in (2, 0, 3, 1):                                 # any order
                ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, 1, w.t_q, path), dtype=torch.uint8,
                                 device="cuda")
                sc = torch.empty((1, w.n_frames), dtype=torch.float32, device="cuda")
                idx = torch.full((1, k), -7, dtype=torch.int32, device="cuda")
                ko = torch.zeros((1, Hk, k * G, d), dtype=torch.bfloat16, device="cuda")
                vo = torch.zeros_like(ko)
                oqm.tom_oqm_score_groups(mem.handle, l, 1, qd[l:l + 1].contiguous(), w.t_q, sc, w.n_frames, None,
                                         path, ws)
                assert oqm.tom_oqm_topk(sc, w.n_frames, 1, w.n_frames, k, idx) == k_eff
                oqm.tom_oqm_dequant_gather(mem.handle, l, 1, idx, k, k_eff, ko, vo)
                torch.cuda.synchronize()
                got = sc.cpu().numpy().astype(np.float64)
                assert np.all(np.abs(got - ref_scores[l:l + 1]) <= H.score_bound(st, q, ref_scores[l:l + 1]))
                assert np.array_equal(idx.cpu().numpy(), ref_idx[l:l + 1])
                assert np.array_equal(H.bits(ko), ref_k[l:l + 1]) and np.array_equal(H.bits(vo), ref_v[l:l + 1])
                # the one-call form on the same single layer
                ko.zero_()
                vo.zero_()
                idx.fill_(-7)
                assert oqm.tom_oqm_retrieve(mem.handle, l, 1, qd[l:l + 1].contiguous(), w.t_q, k, sc, w.n_frames,
                                            idx, ko, vo, ws, path=path) == k_eff
                torch.cuda.synchronize()
                assert np.array_equal(idx.cpu().numpy(), ref_idx[l:l + 1])
                assert np.array_equal(H.bits(ko), ref_k[l:l + 1]) and np.array_equal(H.bits(vo), ref_v[l:l + 1])
    finally:
        mem.close()


def test_random_configurations_sweep(oqm):
    """Seeded random shapes, dtypes, axes, code widths and call patterns, each streamed through
    the whole path and compared with the oracle element by element."""
    rng = np.random.default_rng(20251018)
    for case in range(24):
        d = int(rng.choice([8, 16, 32, 64, 96, 128, 160, 256]))
        gs_all = [g for g in (8, 16, 32, 64, 128) if d % g == 0]
        gs = int(rng.choice(gs_all))
        Hk = int(rng.integers(1, 5))
        r = int(rng.choice([1, 2, 7]))
        G = int(rng.choice([1, 3, 16, 31, 50, 64, 100, 196, 211]))
        L = int(rng.integers(1, 4))
        T = int(rng.integers(3, 20))
        dt = str(rng.choice(["f32", "bf16", "f16"]))
        qaxis = int(rng.integers(0, 2))
        bits = int(rng.choice([4, 2]))
        tq = int(rng.choice([1, 5, 16, 33]))
        k = int(rng.integers(1, T + 3))
        per_call = int(rng.integers(1, T + 1))
        sim = str(rng.choice(["cosine", "dot"]))
        kind = str(rng.choice(["normal", "layer_std", "outlier"]))
        path = oqm.TOM_SCORE_TOKEN_GEMM if rng.integers(0, 2) else None
        meta = str(rng.choice(["f32", "bf16"]))
        w = synth_kv.Workload("R", L, Hk, Hk * r, d, G, T, gs, tq, k, dt, sim, 9000 + case, kind, per_call)
        print(f"case {case}: {w} qaxis={qaxis} bits={bits} path={path} meta={meta}", flush=True)
        res = _stream_and_check(oqm, w, per_call, path=path, want_tokens=path is not None, qaxis=qaxis,
                                bits=bits, meta=meta)
        assert res["k_eff"] == min(k, T)


def test_side_stream_and_graph_replay(oqm):
    """The calls only queue work on the stream they are given: the path on a non-default
    stream, and the one-call retrieval captured into a HIP graph and replayed several times
    with eager work in between, must give what the eager default-stream calls give."""
    w = synth_kv.Workload("X", 3, 4, 28, 128, 50, 40, 64, 8, 6, "bf16", "cosine", 4242, "layer_std", 40)
    st, mem = H.pair_for(oqm, w)
    try:
        L, Hk, G, d, k, T = w.n_layers, w.n_kv_heads, w.group_tokens, w.head_dim, w.top_k, w.n_frames
        kk, vv = synth_kv.kv_frames(w, 0, T)
        H.orc.quantize_append(st, H.bits(kk), H.bits(vv))
        side = torch.cuda.Stream()                               # default priority
        kd, vd = kk.cuda(), vv.cuda()
        qs = [synth_kv.query(w, i).cuda() for i in range(3)]
        scores = torch.empty((L, T), dtype=torch.float32, device="cuda")
        idx = torch.full((L, k), -7, dtype=torch.int32, device="cuda")
        ko = torch.zeros((L, Hk, k * G, d), dtype=torch.bfloat16, device="cuda")
        vo = torch.zeros_like(ko)
        ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, w.t_q, oqm.TOM_SCORE_AUTO),
                         dtype=torch.uint8, device="cuda")
        qbuf = qs[0].clone()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            oqm.tom_oqm_quantize_append(mem.handle, 0, L, T, kd, vd, stream=side.cuda_stream)
            oqm.tom_oqm_retrieve(mem.handle, 0, L, qbuf, w.t_q, k, scores, T, idx, ko, vo, ws,
                                 stream=side.cuda_stream)
        side.synchronize()
        H.compare_storage(st, mem)

        def reference(q):
            sc = H.orc.score_groups(st, H.bits(q), 1)
            ii, k_eff = H.orc.topk(sc, k)
            rk, rv = H.orc.dequant_gather(st, ii, k_eff)
            return ii, rk, rv

        ii, rk, rv = reference(qs[0])
        assert np.array_equal(idx.cpu().numpy(), ii) and np.array_equal(H.bits(ko), rk) and np.array_equal(H.bits(vo), rv)

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            oqm.tom_oqm_retrieve(mem.handle, 0, L, qbuf, w.t_q, k, scores, T, idx, ko, vo, ws,
                                 stream=torch.cuda.current_stream().cuda_stream)
        for rep in range(4):
            q = qs[rep % 3]
            qbuf.copy_(q)                                        # eager work between the replays
            ko.zero_()
            vo.zero_()
            idx.fill_(-7)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ii, rk, rv = reference(q)
            assert np.array_equal(idx.cpu().numpy(), ii), f"replay {rep}"
            assert np.array_equal(H.bits(ko), rk) and np.array_equal(H.bits(vo), rv), f"replay {rep}"
    finally:
        mem.close()


def test_division_shortcuts_are_exact_for_every_input():
    """The quantize kernel computes (max - min) / 15 and 1 / s with one FMA correction step
    instead of the full IEEE division sequence; the library's self-check program compares
    both with IEEE division for all ~2^31 possible inputs on the GPU."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                       "paper_2510_18269_amd", "selfcheck_division.bin")
    assert os.path.exists(exe), "build the library first (python -m paper_2510_18269_amd.build)"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "div15_exact mismatches: 0" in r.stdout and "rcp_exact mismatches: 0" in r.stdout
    assert "div3_exact mismatches: 0" in r.stdout
