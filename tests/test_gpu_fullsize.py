"""GPU parity at the benchmark's full sizes and launch configuration (C3, C4, C5).

The oracle cannot redo 10^10 elements, so it recomputes a SAMPLE of frame-groups one by one
(all layers, heads, K and V of each sampled group) from the same seeded inputs, and the rest is
covered by properties that hold at any size:
  * stored tiles of the sampled groups: codes, scale, zero bit-exact, keys within one ulp;
  * scores of the sampled groups (oracle keys, oracle score) within one float32 ulp;
  * top-k of the GPU's full score rows, recomputed by the oracle, equals the GPU indices;
  * dequant-gather of the sampled groups bit-exact, rows past k_eff*G untouched;
  * every gathered row block of the real retrieval equals the gather of that index alone.
Inputs are generated on the GPU by the seeded generator (the same call reproduces the same bits),
so a sampled batch is simply drawn again and copied to the host for the oracle."""
import numpy as np
import pytest
import torch

import synth_kv
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oqm():
    from paper_2510_18269_amd import oqm as m
    assert torch.cuda.is_available()
    return m


def _oracle_sample(w, sampled_groups, fpa, qaxis=0, bits=4, meta_dtype=0):
    """Oracle store holding only the sampled frame-groups: slot j <-> group sampled_groups[j]."""
    orc = H.orc
    dt = H.DT[w.dtype][0]
    cfg = orc.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens,
                          w.qgroup, len(sampled_groups), qaxis=qaxis, bits=bits, in_dtype=dt, out_dtype=dt,
                          sim=1 if w.sim == "cosine" else 0, meta_dtype=meta_dtype)
    st = orc.new_store(cfg)
    for t in sampled_groups:
        f0 = (t // fpa) * fpa
        k, v = synth_kv.kv_frames(w, f0, fpa, "cuda")            # same seed -> same bits as appended
        kk = k[t - f0:t - f0 + 1].cpu()
        vv = v[t - f0:t - f0 + 1].cpu()
        orc.quantize_append(st, H.bits(kk), H.bits(vv))
        del k, v
    return st


def _compare_sampled_storage(w, st, mem, sampled_groups):
    cfg = st.cfg
    L, Hk, G, d, gs, T = w.n_layers, w.n_kv_heads, w.group_tokens, w.head_dim, w.qgroup, mem.cfg.capacity_groups
    codes = mem.codes.view(L, 2, T, Hk, G, d * cfg.bits // 8)
    meta = mem.meta.view(L, 2, T, Hk, G, d // gs, 2) if cfg.qaxis == 0 else mem.meta.view(L, 2, T, Hk, d, 2)
    if meta.dtype == torch.bfloat16:
        meta = meta.float()                                           # exact widening of the stored pairs
    keys = mem.keys.view(L, T, Hk, d)
    oc, os_, oz, ok = H.storage_views(cfg, st.codes, st.scale, st.zero, st.keys)
    not_identical = 0
    for j, t in enumerate(sampled_groups):
        H._same(codes[:, :, t].cpu().numpy(), oc[:, :, j], f"codes of group {t}")
        m = meta[:, :, t].cpu().numpy()
        H._same(np.ascontiguousarray(m[..., 0]).view(np.uint32), os_[:, :, j].view(np.uint32), f"scale of group {t}")
        H._same(np.ascontiguousarray(m[..., 1]).view(np.uint32), oz[:, :, j].view(np.uint32), f"zero of group {t}")
        gk = keys[:, t].cpu().numpy()
        assert np.all(np.abs(gk - ok[:, j]) <= np.spacing(np.abs(ok[:, j]))), f"keys of group {t}"
        not_identical += int(np.sum(gk != ok[:, j]))
    return not_identical


def _retrieve_and_check(oqm, w, st, mem, sampled_groups, path, q, n_stored):
    orc = H.orc
    L, G = w.n_layers, w.group_tokens
    sc, _ = H.gpu_scores(oqm, mem, q, path)
    sc_np = sc.cpu().numpy()[:, :n_stored]
    assert np.isfinite(sc_np).all() and np.all(np.abs(sc_np) <= 1 + 1e-6)
    # scores of the sampled groups against the oracle (its own keys, float64 accumulation)
    live = [(j, t) for j, t in enumerate(sampled_groups) if t < n_stored]
    ref = orc.score_groups(st, H.bits(q.cpu()), H.DT[w.dtype][0])
    for j, t in live:
        b = np.spacing(np.abs(ref[:, j])).astype(np.float64) + 1e-12
        assert np.all(np.abs(sc_np[:, t].astype(np.float64) - ref[:, j]) <= b), f"score of group {t}"
    # selection: oracle top-k of the GPU's own full rows
    idx, k_eff, ko, vo = H.gpu_retrieve(oqm, mem, sc, w.top_k, L, fill=0x7FC1)
    want, k_ref = orc.topk(np.ascontiguousarray(sc_np), w.top_k)
    assert k_eff == k_ref == min(w.top_k, n_stored)
    assert np.array_equal(idx[:, :k_eff], want[:, :k_eff])
    assert np.all(np.diff(idx[:, :k_eff], axis=1) > 0)               # temporal order
    if k_eff < w.top_k:
        assert np.all(ko[:, :, k_eff * G:] == 0x7FC1) and np.all(vo[:, :, k_eff * G:] == 0x7FC1)
    # reconstruction of the sampled groups, alone, against the oracle
    ks = len(live)
    if ks:
        sidx = torch.tensor([[t for _, t in live]] * L, dtype=torch.int32, device="cuda")
        tdt = mem.out_torch_dtype()
        shape = (L, w.n_kv_heads, ks * G, w.head_dim)
        sk = torch.empty(shape, dtype=tdt, device="cuda")
        sv = torch.empty(shape, dtype=tdt, device="cuda")
        oqm.tom_oqm_dequant_gather(mem.handle, 0, L, sidx, ks, ks, sk, sv)
        torch.cuda.synchronize()
        oidx = np.array([[j for j, _ in live]] * L, np.int32)
        rk, rv = orc.dequant_gather(st, oidx, ks)
        assert np.array_equal(H.bits(sk), rk) and np.array_equal(H.bits(sv), rv)
        # the real retrieval wrote the same bytes wherever it picked a sampled group
        skb, svb = H.bits(sk), H.bits(sv)
        hits = 0
        for l in range(L):
            for r in range(k_eff):
                for pos, (_, t) in enumerate(live):
                    if idx[l, r] == t:
                        assert np.array_equal(ko[l, :, r * G:(r + 1) * G], skb[l, :, pos * G:(pos + 1) * G])
                        assert np.array_equal(vo[l, :, r * G:(r + 1) * G], svb[l, :, pos * G:(pos + 1) * G])
                        hits += 1
        return hits
    return 0


@pytest.mark.parametrize("name", ["C3", "C5"])
def test_bulk_stream_full_size(oqm, name):
    w = synth_kv.WORKLOADS[name]
    fpa = w.frames_per_append
    cfg = oqm.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens, w.qgroup,
                          w.n_frames, in_dtype=1, out_dtype=1, sim=oqm.TOM_SIM_COSINE)
    mem = oqm.Memory.allocate(cfg)
    try:
        for f0 in range(0, w.n_frames, fpa):
            k, v = synth_kv.kv_frames(w, f0, fpa, "cuda")
            first = oqm.tom_oqm_quantize_append(mem.handle, 0, w.n_layers, fpa, k, v)
            assert first == f0
            torch.cuda.synchronize()
            del k, v
        assert mem.n_groups == w.n_frames
        sampled = [0, 31, 32, 333, 500, 777, 1000, w.n_frames - 1]
        st = _oracle_sample(w, sampled, fpa)
        diff = _compare_sampled_storage(w, st, mem, sampled)
        assert diff <= 2                                              # keys practically identical
        path = oqm.TOM_SCORE_TOKEN_GEMM if name == "C5" else oqm.TOM_SCORE_MEAN_QUERY
        q = synth_kv.query(w, 0, "cuda")
        _retrieve_and_check(oqm, w, st, mem, sampled, path, q, w.n_frames)
        # a query that IS a stored summary key retrieves its group in every layer
        keys = mem.keys.view(w.n_layers, w.n_frames, w.n_kv_heads, 1, w.head_dim)
        r = w.n_q_heads // w.n_kv_heads
        planted = keys[:, 777].repeat_interleave(r, dim=1).expand(-1, -1, w.t_q, -1).contiguous()
        sc, _ = H.gpu_scores(oqm, mem, planted, path)
        assert (sc[:, :w.n_frames].argmax(1) == 777).all()
        assert torch.allclose(sc[:, 777], torch.ones(w.n_layers, device="cuda"), atol=1e-6)
    finally:
        mem.close()


@pytest.mark.parametrize("G,dt,qaxis,bits,meta", [
    (50, "f16", 1, 4, "f32"),       # the paper's own setting (Eq. 9, 50 tokens, FP16)
    (196, "bf16", 0, 2, "f32"),     # 2-bit ablation at the benchmark's shape
    (50, "f16", 1, 2, "f32"),
    (196, "bf16", 0, 4, "bf16"),    # bfloat16 (scale, zero) pairs at the benchmark's shape
    (50, "f16", 1, 4, "bf16")])
def test_variants_full_size(oqm, G, dt, qaxis, bits, meta):
    """The 1024-frame, 28-layer stream with the token-axis quantizer and / or 2-bit codes."""
    w = synth_kv.scaled(synth_kv.WORKLOADS["C3"], group_tokens=G, dtype=dt)
    fpa = w.frames_per_append
    dtc = H.DT[dt][0]
    cfg = oqm.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, G, w.qgroup, w.n_frames,
                          qaxis=qaxis, bits=bits, in_dtype=dtc, out_dtype=dtc, sim=oqm.TOM_SIM_COSINE,
                          meta_dtype=H.DT[meta][0])
    mem = oqm.Memory.allocate(cfg)
    try:
        for f0 in range(0, w.n_frames, fpa):
            k, v = synth_kv.kv_frames(w, f0, fpa, "cuda")
            oqm.tom_oqm_quantize_append(mem.handle, 0, w.n_layers, fpa, k, v)
            torch.cuda.synchronize()
            del k, v
        sampled = [0, 31, 32, 500, 1000, w.n_frames - 1]
        st = _oracle_sample(w, sampled, fpa, qaxis, bits, H.DT[meta][0])
        assert _compare_sampled_storage(w, st, mem, sampled) <= 2
        _retrieve_and_check(oqm, w, st, mem, sampled, oqm.TOM_SCORE_MEAN_QUERY, synth_kv.query(w, 0, "cuda"),
                            w.n_frames)
    finally:
        mem.close()


def test_hour_long_stream_one_frame_per_append(oqm):
    """C4: 3600 frames appended one at a time, a query every 36 frames (100 queries)."""
    w = synth_kv.WORKLOADS["C4"]
    cfg = oqm.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens, w.qgroup,
                          w.n_frames, in_dtype=1, out_dtype=1, sim=oqm.TOM_SIM_COSINE)
    mem = oqm.Memory.allocate(cfg)
    sampled = [0, 35, 36, 1234, 2500, 3599]
    st = _oracle_sample(w, sampled, 1)
    try:
        n_queries = 0
        hits = 0
        for f in range(w.n_frames):
            k, v = synth_kv.kv_frames(w, f, 1, "cuda")
            oqm.tom_oqm_quantize_append(mem.handle, 0, w.n_layers, 1, k, v)
            if (f + 1) % 36 == 0:
                n_queries += 1
                full = n_queries in (1, 2, 50, 100)
                q = synth_kv.query(w, n_queries, "cuda")
                if full:
                    hits += _retrieve_and_check(oqm, w, st, mem, sampled, oqm.TOM_SCORE_MEAN_QUERY, q, f + 1)
                else:                                                 # selection property only
                    sc, _ = H.gpu_scores(oqm, mem, q, oqm.TOM_SCORE_MEAN_QUERY)
                    idx, k_eff, _, _ = H.gpu_retrieve(oqm, mem, sc, w.top_k, w.n_layers)
                    want, _ = H.orc.topk(np.ascontiguousarray(sc.cpu().numpy()[:, :f + 1]), w.top_k)
                    assert k_eff == min(w.top_k, f + 1) and np.array_equal(idx[:, :k_eff], want[:, :k_eff])
        torch.cuda.synchronize()
        assert n_queries == 100 and mem.n_groups == 3600
        assert _compare_sampled_storage(w, st, mem, sampled) <= 2
        with pytest.raises(oqm.TomError) as e:                        # the store is full: nothing is evicted
            oqm.tom_oqm_quantize_append(mem.handle, 0, w.n_layers, 1, k, v)
        assert e.value.status == oqm.TOM_ERR_CAPACITY
    finally:
        mem.close()
