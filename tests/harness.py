"""Drives the CPU oracle and the GPU library side by side on the same seeded inputs.
Used by the GPU parity tests; holds comparison logic only (no arithmetic of the method)."""
from __future__ import annotations

import numpy as np
import torch

import synth_kv
from oracle import oqm_oracle as orc

DT = {  # name -> (oracle/ABI dtype code, torch dtype)
    "f32": (0, torch.float32), "bf16": (1, torch.bfloat16), "f16": (2, torch.float16)}


def bits(t: torch.Tensor) -> np.ndarray:
    return synth_kv.as_numpy_bits(t)


def make_pair(oqm, *, n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup, capacity,
              in_dtype="bf16", out_dtype=None, sim="cosine", qaxis=0, bits=4, meta="f32"):
    out_dtype = out_dtype or in_dtype
    simc = 1 if sim == "cosine" else 0
    ocfg = orc.make_config(n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup,
                           capacity, qaxis=qaxis, bits=bits, in_dtype=DT[in_dtype][0],
                           out_dtype=DT[out_dtype][0], sim=simc, meta_dtype=DT[meta][0])
    gcfg = oqm.make_config(n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup,
                           capacity, qaxis=qaxis, bits=bits, in_dtype=DT[in_dtype][0],
                           out_dtype=DT[out_dtype][0], sim=simc, meta_dtype=DT[meta][0])
    return orc.new_store(ocfg), oqm.Memory.allocate(gcfg)


def pair_for(oqm, w: synth_kv.Workload, capacity=None, out_dtype=None, qaxis=0, bits=4, meta="f32"):
    return make_pair(oqm, n_layers=w.n_layers, n_kv_heads=w.n_kv_heads, n_q_heads=w.n_q_heads,
                     head_dim=w.head_dim, group_tokens=w.group_tokens, qgroup=w.qgroup,
                     capacity=capacity or w.n_frames, in_dtype=w.dtype, out_dtype=out_dtype,
                     sim=w.sim, qaxis=qaxis, bits=bits, meta=meta)


def append_both(oqm, st, mem, k: torch.Tensor, v: torch.Tensor, ksum: torch.Tensor | None = None):
    """k, v: CPU tensors [F][L][H][G][d]; appended to both sides (all layers)."""
    F, L = k.shape[0], k.shape[1]
    orc.quantize_append(st, bits(k), bits(v), None if ksum is None else bits(ksum))
    kd, vd = k.cuda(), v.cuda()
    sd = None if ksum is None else ksum.cuda()
    oqm.tom_oqm_quantize_append(mem.handle, 0, L, F, kd, vd, sd)
    torch.cuda.synchronize()


def storage_views(cfg, codes, scale, zero, keys):
    """Reshape flat storage arrays to [L][2][T_cap][...] / [L][T_cap][...]."""
    L, T, H, G, d, gs = (cfg.n_layers, cfg.capacity_groups, cfg.n_kv_heads, cfg.group_tokens,
                         cfg.head_dim, cfg.qgroup)
    mshape = (L, 2, T, H, G, d // gs) if cfg.qaxis == 0 else (L, 2, T, H, d)
    return (codes.reshape(L, 2, T, H, G, d * cfg.bits // 8), scale.reshape(mshape), zero.reshape(mshape),
            keys.reshape(L, T, H, d))


def _same(got: np.ndarray, want: np.ndarray, what: str):
    """Bit-exact comparison that names the first mismatch ([L][K|V][t][h][token][...])."""
    if np.array_equal(got, want):
        return
    bad = np.argwhere(got != want)
    first = tuple(int(i) for i in bad[0])
    raise AssertionError(f"{what} differ in {len(bad)} of {got.size} entries; first at {first}: "
                         f"gpu {got[first]:#x} oracle {want[first]:#x}")


def compare_storage(st, mem, lo=0, hi=None, key_abs=None):
    """Codes, scale, zero bit-exact; summary keys within one float32 ulp (float64 sums
    rounded once on both sides, so they are almost always identical).  `key_abs`
    ([L][T_cap][H] array) widens the key tolerance per tile to that absolute value: for
    tiles whose columns cancel across more of the float64 range than a sum keeps, where
    the order of the additions shows (pass 1e-6 * max|K| of the tile)."""
    cfg = st.cfg
    hi = st.n_groups if hi is None else hi
    assert mem.n_groups == st.n_groups
    oc, os_, oz, ok = storage_views(cfg, st.codes, st.scale, st.zero, st.keys)
    if mem.meta.dtype == torch.bfloat16:                 # widen the stored bfloat16 pairs (exact)
        meta = (bits(mem.meta).astype(np.uint32) << 16).view(np.float32).reshape(-1, 2)
    else:
        meta = mem.meta.cpu().numpy().reshape(-1, 2)     # (scale, zero) pairs
    gc, gs_, gz, gk = storage_views(cfg, mem.codes.cpu().numpy(), np.ascontiguousarray(meta[:, 0]),
                                    np.ascontiguousarray(meta[:, 1]), mem.keys.cpu().numpy())
    sl = slice(lo, hi)
    _same(gc[:, :, sl], oc[:, :, sl], "packed codes")
    _same(gs_[:, :, sl].view(np.uint32), os_[:, :, sl].view(np.uint32), "scale")
    _same(gz[:, :, sl].view(np.uint32), oz[:, :, sl].view(np.uint32), "zero")
    a, b = gk[:, sl], ok[:, sl]
    ulp = np.spacing(np.abs(b).astype(np.float32)).astype(np.float64)
    if key_abs is not None:
        ulp = np.maximum(ulp, np.asarray(key_abs, np.float64)[:, sl, :, None])
    assert np.all(np.abs(a.astype(np.float64) - b) <= ulp), "summary keys differ by more than the bound"
    return float(np.mean(a != b))      # fraction of keys not bit-identical


def gpu_scores(oqm, mem, q: torch.Tensor, path=None, want_tokens=False, layer0=0, n_layers=None,
               stride_pad=0):
    cfg = mem.cfg
    nl = q.shape[0] if n_layers is None else n_layers
    tq = q.shape[2]
    T = mem.n_groups
    path = oqm.TOM_SCORE_AUTO if path is None else path
    stride = T + stride_pad
    scores = torch.full((nl, max(stride, 1)), float("nan"), dtype=torch.float32, device="cuda")
    tok = torch.full((nl, tq, T), float("nan"), dtype=torch.float32, device="cuda") if want_tokens else None
    nbytes = oqm.tom_oqm_score_workspace_bytes(mem.handle, nl, tq, path, want_tokens)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    oqm.tom_oqm_score_groups(mem.handle, layer0, nl, q.cuda(), tq, scores, stride, tok, path, ws)
    torch.cuda.synchronize()
    return scores, tok


def score_bound(st, q: torch.Tensor, scores_ref: np.ndarray) -> np.ndarray:
    """What the GPU score may differ from the oracle's by: both accumulate in float64 and
    round once to float32, so one float32 ulp of the score (plus a denormal floor)."""
    floor = 1e-12 * np.maximum(1.0, np.abs(scores_ref).max(axis=-1, keepdims=True))
    return np.spacing(np.abs(scores_ref).astype(np.float32)).astype(np.float64) + floor


def check_indices(gpu_idx: np.ndarray, gpu_scores_np: np.ndarray, ref_scores: np.ndarray, k: int,
                  bound: np.ndarray, order=0):
    """(i) top-k of the GPU's own scores, recomputed by the oracle, must equal the GPU's
    indices bit for bit.  (ii) against the oracle's scores: identical whenever the margin
    between the k-th and (k+1)-th oracle score exceeds twice the score tolerance; otherwise
    every chosen score must reach the boundary minus the tolerance."""
    rows, T = ref_scores.shape
    want, k_eff = orc.topk(np.ascontiguousarray(gpu_scores_np[:, :T]), k, order)
    assert np.array_equal(gpu_idx[:, :k_eff], want[:, :k_eff]), "top-k of the GPU's own scores differs"
    ref_idx, _ = orc.topk(ref_scores, k, order)
    n_loose = 0
    for r in range(rows):
        if np.array_equal(gpu_idx[r, :k_eff], ref_idx[r, :k_eff]):
            continue
        srt = np.sort(ref_scores[r])[::-1]
        margin = srt[k_eff - 1] - srt[k_eff] if k_eff < T else np.inf
        tol = 2 * float(bound[r].max())
        assert margin <= tol, f"row {r}: indices differ although the margin {margin} > {tol}"
        chosen = ref_scores[r, gpu_idx[r, :k_eff]]
        assert np.all(chosen >= srt[k_eff - 1] - tol)
        n_loose += 1
    return k_eff, n_loose


def gpu_retrieve(oqm, mem, scores: torch.Tensor, k: int, n_layers: int, order=0, guard_rows=0,
                 fill=None):
    """top-k + dequant-gather on the GPU.  Returns (idx [L][k] np, k_eff, K_act, V_act np bits)."""
    cfg = mem.cfg
    T = mem.n_groups
    idx = torch.full((n_layers, k), -7, dtype=torch.int32, device="cuda")
    k_eff = oqm.tom_oqm_topk(scores, scores.shape[1], n_layers, T, k, idx, order)
    rows = k * cfg.group_tokens + guard_rows
    tdt = mem.out_torch_dtype()
    shape = (n_layers, cfg.n_kv_heads, k * cfg.group_tokens, cfg.head_dim)
    ko = torch.empty(shape, dtype=tdt, device="cuda")
    vo = torch.empty(shape, dtype=tdt, device="cuda")
    if fill is not None:
        ko.view(torch.int16 if tdt != torch.float32 else torch.int32).fill_(fill)
        vo.view(torch.int16 if tdt != torch.float32 else torch.int32).fill_(fill)
    oqm.tom_oqm_dequant_gather(mem.handle, 0, n_layers, idx, k, k_eff, ko, vo)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), k_eff, bits(ko), bits(vo)


def full_path_check(oqm, st, mem, q: torch.Tensor, k: int, path=None, want_tokens=False):
    """score -> top-k -> dequant-gather on both sides; asserts the parity bar.  Returns stats."""
    cfg = st.cfg
    nl = q.shape[0]
    qdt = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[q.dtype]
    ref = orc.score_groups(st, bits(q), qdt, want_token_scores=want_tokens)
    ref_scores, ref_tok = ref if want_tokens else (ref, None)
    sc, tok = gpu_scores(oqm, mem, q, path, want_tokens)
    sc_np = sc.cpu().numpy()
    bound = score_bound(st, q, ref_scores)
    assert np.all(np.abs(sc_np[:, :st.n_groups].astype(np.float64) - ref_scores) <= bound), \
        "scores differ from the oracle"
    frac_score_equal = float(np.mean(sc_np[:, :st.n_groups] == ref_scores))
    if want_tokens:
        tb = np.spacing(np.abs(ref_tok).astype(np.float32)).astype(np.float64) \
            + 1e-12 * max(1.0, float(np.abs(ref_tok).max()))
        assert np.all(np.abs(tok.cpu().numpy().astype(np.float64) - ref_tok) <= tb), \
            "per-token scores differ"
    fillv = 0x7FC1 if cfg.out_dtype != 0 else 0x7FC00001
    idx, k_eff, ko, vo = gpu_retrieve(oqm, mem, sc, k, nl, fill=fillv)
    k_eff2, n_loose = check_indices(idx, sc_np, ref_scores, k, bound)
    assert k_eff2 == k_eff == min(k, st.n_groups)
    # values: the oracle dequantizes ITS store at the GPU's indices (identical to its own
    # indices except on documented near-ties); bit-exact compare, which implies the
    # stated 1e-6 relative / 1 bf16 ulp tolerance
    idx_fill = idx.copy()
    ok_ref, ov_ref = orc.dequant_gather(st, idx_fill, k_eff, fill=(fillv & 0xFFFF) if cfg.out_dtype != 0 else None)
    if cfg.out_dtype == 0:
        G = cfg.group_tokens
        assert np.array_equal(ko[:, :, :k_eff * G].view(np.uint32), ok_ref[:, :, :k_eff * G].view(np.uint32))
        assert np.array_equal(vo[:, :, :k_eff * G].view(np.uint32), ov_ref[:, :, :k_eff * G].view(np.uint32))
        if k_eff < k:
            assert np.all(ko[:, :, k_eff * G:].view(np.uint32) == fillv)
            assert np.all(vo[:, :, k_eff * G:].view(np.uint32) == fillv)
    else:
        assert np.array_equal(ko, ok_ref), "active K differs"
        assert np.array_equal(vo, ov_ref), "active V differs"
    return dict(k_eff=k_eff, loose_rows=n_loose, frac_score_equal=frac_score_equal)
