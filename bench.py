#!/usr/bin/env python3
"""Benchmark of the OQM hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
    quantize-append of `frames_per_append` frames (all layers, K and V)
    -> score all stored frame-groups against a T_q-token query
    -> top-k per layer -> dequant-gather of the k groups into the bf16 active KV buffer.
All inputs are resident in HBM before the timed region.  The store is pre-filled, and every
step overwrites a rotating window of group slots so that it always holds the full stream.

Prints ONE JSON line (see README / DESIGN notes for the field meanings).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
METRIC = "OQM quantize-append + retrieve/dequant HBM GB/s (% of peak); retrieval ms/query"


def bytes_append(w, n_frames, in_bytes, bits=4, meta_b=8):
    e = n_frames * w.n_layers * 2 * w.n_kv_heads * w.group_tokens * w.head_dim
    keys = n_frames * w.n_layers * w.n_kv_heads * w.head_dim * 4
    return e * in_bytes + e * bits // 8 + (e // w.qgroup) * meta_b + keys, e


def bytes_gather(w, k_eff, out_bytes, bits=4, meta_b=8):
    e = w.n_layers * k_eff * 2 * w.n_kv_heads * w.group_tokens * w.head_dim
    return e * bits // 8 + (e // w.qgroup) * meta_b + e * out_bytes + w.n_layers * k_eff * 4, e


def bytes_score(w, T, q_bytes):
    hd = w.n_kv_heads * w.head_dim
    return w.n_layers * T * hd * 4 + w.n_layers * w.n_q_heads * w.t_q * w.head_dim * q_bytes + w.n_layers * T * 4


def bytes_topk(w, T, k_eff):
    return w.n_layers * T * 4 + w.n_layers * k_eff * 4


def measured_traffic(kernel, workload):
    """HBM bytes per launch (read + written) of `kernel`, from the committed rocprofv3
    FETCH_SIZE / WRITE_SIZE summary of this same command, or None if there is none."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_bench_{workload.lower()}.txt")
    try:
        with open(path) as f:
            for line in f:
                p = line.split()
                if len(p) == 5 and p[0] == "traffic" and p[1] == kernel and p[2] == workload:
                    return int(p[3]) + int(p[4])
    except OSError:
        pass
    return None


def load_probe_lib():
    """The benchmark-only shared object (stream probes, timing events); not part of the library."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2510_18269_amd", "libtom_bench_probe.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build first (python -m paper_2510_18269_amd.build)")
    lib = C.CDLL(path)
    lib.bench_stream_probe.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.bench_stream_probe.restype = C.c_int
    lib.bench_event_create.argtypes = [C.c_int32]
    lib.bench_event_create.restype = C.c_void_p
    lib.bench_event_record.argtypes = [C.c_void_p, C.c_void_p]
    lib.bench_event_record.restype = C.c_int
    lib.bench_event_synchronize.argtypes = [C.c_void_p]
    lib.bench_event_synchronize.restype = C.c_int
    lib.bench_event_elapsed_ms.argtypes = [C.c_void_p, C.c_void_p]
    lib.bench_event_elapsed_ms.restype = C.c_float
    lib.bench_event_destroy.argtypes = [C.c_void_p]
    lib.bench_event_destroy.restype = None
    return lib


def cpu_baseline(w, batches_cpu, q_cpu, threads, qaxis=0, bits=4, meta="f32"):
    """The oracle, as it stands, on a bounded sample of the same workload: the given append
    batches (all layers) and one retrieval over what they stored.  Threads split layers."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import synth_kv
    from oracle import oqm_oracle as orc

    dt = {"f32": 0, "bf16": 1, "f16": 2}[w.dtype]
    F = sum(b[0].shape[0] for b in batches_cpu)
    cfg = orc.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens,
                          w.qgroup, F, qaxis=qaxis, bits=bits, in_dtype=dt, out_dtype=dt,
                          sim=1 if w.sim == "cosine" else 0, meta_dtype=1 if meta == "bf16" else 0)
    st = orc.new_store(cfg)
    L = w.n_layers
    threads = max(1, min(threads, L))
    kb = [(synth_kv.as_numpy_bits(k), synth_kv.as_numpy_bits(v)) for k, v in batches_cpu]
    qb = synth_kv.as_numpy_bits(q_cpu)
    H, G, d = w.n_kv_heads, w.group_tokens, w.head_dim
    strides = (L * H * G * d, H * G * d, G * d, d)
    k_eff = min(w.top_k, F)
    scores = np.zeros((L, F), np.float32)
    idx = np.zeros((L, w.top_k), np.int32)
    kout = np.zeros((L, H, w.top_k * G, d), np.uint16 if dt else np.float32)
    vout = np.zeros_like(kout)

    def layer_job(l):
        first = 0
        for k, v in kb:
            nf = k.shape[0]
            st_l = orc.Store(st.cfg, st.codes, st.scale, st.zero, st.keys, first)
            orc.quantize_append(st_l, k.ravel()[l * strides[1]:], v.ravel()[l * strides[1]:], None,
                                layer0=l, strides=strides, n_frames=nf, n_layers=1)
            first += nf
        st_l = orc.Store(st.cfg, st.codes, st.scale, st.zero, st.keys, F)
        s = orc.score_groups(st_l, qb[l:l + 1], dt, layer0=l, n_layers=1)
        scores[l] = s[0]
        ii, _ = orc.topk(s, w.top_k)
        idx[l] = ii[0]
        ko, vo = orc.dequant_gather(st_l, ii, k_eff, layer0=l)
        kout[l], vout[l] = ko[0], vo[0]

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(layer_job, range(L)))
    dtm = time.perf_counter() - t0
    t0 = time.perf_counter()
    layer_job(0)                        # the same work for one layer on one thread
    dt1 = time.perf_counter() - t0
    eb = 4 if w.dtype == "f32" else 2
    mb = 4 if meta == "bf16" else 8
    ba, ea = bytes_append(w, F, eb, bits, mb)
    bg, eg = bytes_gather(w, k_eff, eb, bits, mb)
    total = ba + bg + bytes_score(w, F, eb) + bytes_topk(w, F, k_eff)
    return {"value": total / dtm / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{F} frames x {L} layers appended ({len(kb)} calls) + 1 query "
                      f"(T_q={w.t_q}) scored over {F} groups, top-{k_eff} dequant-gathered; "
                      f"{ea + eg} K/V elements in {dtm:.2f} s",
            "one_core": {"value": total / L / dt1 / 1e9, "unit": "GB/s",
                         "sample": f"layer 0 of the same sample on one thread, {dt1:.2f} s"},
            "seconds": dtm}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "C4", "C5", "P64"],
                    help="P64 = the 64-frame stream of the paper's latency breakdown (context figures)")
    ap.add_argument("--frames-per-append", type=int, default=0, help="override the workload's batch")
    ap.add_argument("--qaxis", default=None, choices=["head_dim", "tokens"],
                    help="tokens = the paper's Eq. 9 (scale/zero per channel over the G tokens)")
    ap.add_argument("--group-tokens", type=int, default=0, help="override G (the paper keeps 50)")
    ap.add_argument("--bits", type=int, default=4, choices=[4, 2], help="code width (2 = the paper's ablation)")
    ap.add_argument("--meta", default="f32", choices=["f32", "bf16"],
                    help="precision scale / zero are kept in (bf16 = storage variant, half the metadata)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-batches", type=int, default=32,
                    help="append calls the oracle is timed on (32 x 32 frames = the whole C3 stream)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import synth_kv
    from paper_2510_18269_amd import oqm          # raises if the HIP library is missing

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = synth_kv.WORKLOADS[args.workload]
    if args.qaxis is None:      # the paper's own stream is quantized the paper's way (Eq. 9)
        args.qaxis = "tokens" if args.workload == "P64" else "head_dim"
    if args.group_tokens:
        w = synth_kv.scaled(w, group_tokens=args.group_tokens)
    tok = args.qaxis == "tokens"
    fpa = args.frames_per_append or (w.frames_per_append if w.frames_per_append > 1 else 1)
    fpa = min(fpa, w.n_frames)
    T = (w.n_frames // fpa) * fpa
    eb = 4 if w.dtype == "f32" else 2
    dtc = {"f32": oqm.TOM_F32, "bf16": oqm.TOM_BF16, "f16": oqm.TOM_F16}[w.dtype]
    cfg = oqm.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens,
                          w.qgroup, T, qaxis=oqm.TOM_QAXIS_TOKENS if tok else oqm.TOM_QAXIS_HEAD_DIM,
                          bits=args.bits, in_dtype=dtc, out_dtype=dtc,
                          meta_dtype=oqm.TOM_BF16 if args.meta == "bf16" else oqm.TOM_F32,
                          sim=oqm.TOM_SIM_COSINE if w.sim == "cosine" else oqm.TOM_SIM_DOT)
    mem = oqm.Memory.allocate(cfg, dev)
    if tok:   # byte model: one (scale, zero) pair per channel and tile instead of per gs elements
        w = synth_kv.scaled(w, qgroup=w.group_tokens)
    L = w.n_layers

    # distinct input batches, more than the 256 MB last-level cache can hold, rotated per step
    meta_b = 4 if args.meta == "bf16" else 8
    batch_bytes = bytes_append(w, fpa, eb, args.bits, meta_b)[0]
    n_batches = max(2, min(T // fpa, int(3.0e9 // max(batch_bytes, 1)) or 1, 64))
    batches = [synth_kv.kv_frames(w, i * fpa, fpa, dev) for i in range(n_batches)]
    queries = [synth_kv.query(w, i, dev) for i in range(4)]
    path = oqm.TOM_SCORE_TOKEN_GEMM if args.workload == "C5" else oqm.TOM_SCORE_MEAN_QUERY
    ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, w.t_q, path), dtype=torch.uint8,
                     device=dev)
    scores = torch.zeros((L, T), dtype=torch.float32, device=dev)
    idx = torch.zeros((L, w.top_k), dtype=torch.int32, device=dev)
    tdt = synth_kv.torch_dtype(w)
    outs = [(torch.empty((L, w.n_kv_heads, w.top_k * w.group_tokens, w.head_dim), dtype=tdt, device=dev),
             torch.empty((L, w.n_kv_heads, w.top_k * w.group_tokens, w.head_dim), dtype=tdt, device=dev))
            for _ in range(2)]
    k_eff = min(w.top_k, T)

    # pre-fill the whole store (untimed)
    for i in range(T // fpa):
        k, v = batches[i % n_batches]
        oqm.tom_oqm_quantize_append(mem.handle, 0, L, fpa, k, v)
    torch.cuda.synchronize()
    assert mem.n_groups == T

    n_windows = T // fpa

    def step(i, ev=None):
        """One pass of the hot path.  Plain steps queue two library calls (append, then the
        one-call retrieval = score + top-k + gather back to back); every `EVENT_EVERY`-th step
        takes the same kernels through the separate calls with a HIP event after each, which is
        where the per-kernel durations come from (an event between two kernels costs the
        stream about 5 us, so it is not paid on every step)."""
        k, v = batches[i % n_batches]
        oqm.tom_oqm_set_num_groups(mem.handle, (i % n_windows) * fpa)
        if ev:
            ev[0].record()
        oqm.tom_oqm_quantize_append(mem.handle, 0, L, fpa, k, v)
        if ev:
            ev[1].record()
        oqm.tom_oqm_set_num_groups(mem.handle, T)
        q = queries[i % len(queries)]
        ko, vo = outs[i % 2]
        if not ev:
            oqm.tom_oqm_retrieve(mem.handle, 0, L, q, w.t_q, w.top_k, scores, T, idx, ko, vo, ws, path=path)
            return
        oqm.tom_oqm_score_groups(mem.handle, 0, L, q, w.t_q, scores, T, None, path, ws)
        ev[2].record()
        oqm.tom_oqm_topk(scores, T, L, T, w.top_k, idx)
        ev[3].record()
        oqm.tom_oqm_dequant_gather(mem.handle, 0, L, idx, w.top_k, k_eff, ko, vo)
        ev[4].record()

    # reference: a plain device-to-device copy of known size (1 GiB read + 1 GiB written),
    # untimed part of the run; also the calibration kernel for the HBM byte counters
    copy_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    copy_dst = torch.empty_like(copy_src)
    cev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(2):
        copy_dst.copy_(copy_src)
    cev[0].record()
    for _ in range(5):
        copy_dst.copy_(copy_src)
    cev[1].record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * copy_src.numel() * 4 / (cev[0].elapsed_time(cev[1]) * 1e-3) / 1e9
    del copy_src, copy_dst

    # what the machine reaches for the byte mix of the two big kernels: the library's
    # arithmetic-free stream probes over rotating regions far larger than the last-level cache
    probe_lib = load_probe_lib()

    def probe(mode, read_b, write_b):
        items = 44 << 20
        n_src, n_dst = (12, 4) if read_b < write_b else (4, 12)
        src = torch.empty(items * read_b * n_src, dtype=torch.uint8, device=dev).random_()
        dst = torch.empty(items * write_b * n_dst, dtype=torch.uint8, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = 12
        for i in range(3 + reps):
            if i == 3:
                ev[0].record()
            rc = probe_lib.bench_stream_probe(mode, src.data_ptr() + (i % n_src) * items * read_b,
                                              dst.data_ptr() + (i % n_dst) * items * write_b, items,
                                              torch.cuda.current_stream().cuda_stream)
            assert rc == 0, f"stream probe: hipError {rc}"
        ev[1].record()
        torch.cuda.synchronize()
        return reps * items * (read_b + write_b) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9

    probe_gather = probe(0, 4, 16)
    probe_append = probe(1, 16, 4)
    torch.cuda.empty_cache()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    EVENT_EVERY = 8
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] if i % EVENT_EVERY == 0 else None
              for i in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    events = [e for e in events if e]

    # latency of the one-call retrieval alone: 20 queries back to back between two events
    rev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    rev[0].record()
    for i in range(20):
        ko, vo = outs[i % 2]
        oqm.tom_oqm_retrieve(mem.handle, 0, L, queries[i % len(queries)], w.t_q, w.top_k, scores, T, idx, ko, vo,
                             ws, path=path)
    rev[1].record()
    torch.cuda.synchronize()
    ms_retrieve_call = rev[0].elapsed_time(rev[1]) / 20

    # what an empty interval between two events reads: an upper bound of the events' own cost,
    # which every per-kernel figure below includes (it matters for the short kernels)
    oev = [torch.cuda.Event(enable_timing=True) for _ in range(21)]
    for e in oev:
        e.record()
    torch.cuda.synchronize()
    event_overhead_us = sum(oev[i].elapsed_time(oev[i + 1]) for i in range(20)) / 20 * 1e3

    def avg_ms(a, b):
        return sum(e[a].elapsed_time(e[b]) for e in events) / len(events)

    ms_append, ms_score, ms_topk, ms_gather = avg_ms(0, 1), avg_ms(1, 2), avg_ms(2, 3), avg_ms(3, 4)
    ms_step = wall * 1e3 / args.steps
    b_app, e_app = bytes_append(w, fpa, eb, args.bits, meta_b)
    b_gat, e_gat = bytes_gather(w, k_eff, eb, args.bits, meta_b)
    default_variant = (not tok and args.bits == 4 and not args.group_tokens and not args.frames_per_append
                       and args.meta == "f32")
    b_sc, b_tk = bytes_score(w, T, eb), bytes_topk(w, T, k_eff)
    total_bytes = b_app + b_gat + b_sc + b_tk
    gbps = lambda b, ms: b / (ms * 1e-3) / 1e9
    tokens_per_append = fpa * w.group_tokens

    out = {
        "metric": METRIC,
        "value": round(gbps(total_bytes, ms_step), 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"{w.name}: {L} layers, {w.n_kv_heads} KV heads ({w.n_q_heads} query heads), "
                        f"head_dim {w.head_dim}, {w.dtype} K/V, {T} frames x {w.group_tokens} tokens stored, "
                        f"{fpa} frames per quantize-append, {args.bits}-bit codes, {args.meta} scale/zero, "
                        + (f"scale/zero per channel over the {w.group_tokens} tokens, " if tok else
                           f"quant-group {w.qgroup} over head_dim, ") +
                        ""
                        f"{w.t_q}-token query, top-{k_eff} groups dequant-gathered to {w.dtype}",
            "value_recipe": w.kind, "score_path": "token_gemm" if path == oqm.TOM_SCORE_TOKEN_GEMM else "mean_query",
            "input_batches_rotated": n_batches, "steps_with_kernel_events": len(events),
        },
        "pct_of_hbm_peak": round(100 * gbps(total_bytes, ms_step) / HBM_PEAK_GBPS, 2),
        "copy_GBps": round(copy_gbps, 1),
        "probe": {"gather_mix_GBps": round(probe_gather, 1), "append_mix_GBps": round(probe_append, 1),
                  "what": "arithmetic-free linear streams of the library with the kernels' read/write "
                          "mix (4 B in / 16 B out, 16 B in / 4 B out), same run"},
        "bytes_per_step": total_bytes,
        "append": {"ms": round(ms_append, 4), "GBps": round(gbps(b_app, ms_append), 1),
                   "pct_of_peak": round(100 * gbps(b_app, ms_append) / HBM_PEAK_GBPS, 2),
                   "tokens_per_s": round(tokens_per_append / (ms_append * 1e-3), 1), "bytes": b_app},
        "score": {"ms": round(ms_score, 4), "GBps": round(gbps(b_sc, ms_score), 1), "bytes": b_sc},
        "topk": {"ms": round(ms_topk, 4)},
        "gather": {"ms": round(ms_gather, 4), "GBps": round(gbps(b_gat, ms_gather), 1),
                   "pct_of_peak": round(100 * gbps(b_gat, ms_gather) / HBM_PEAK_GBPS, 2), "bytes": b_gat},
        "event_overhead_us": round(event_overhead_us, 2),
        "retrieval_ms_per_query": round(ms_retrieve_call, 4),
        "retrieval_ms_per_query_separate_calls": round(ms_score + ms_topk + ms_gather, 4),
        "roofline": {"bound": "hbm", "kernel": "dequant_gather_kernel",
                     "achieved": round(gbps(b_gat, ms_gather), 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps(b_gat, ms_gather) / HBM_PEAK_GBPS, 4),
                     "frac_of_probe": round(gbps(b_gat, ms_gather) / probe_gather, 4),
                     "traffic": measured_traffic("dequant_gather_kernel", w.name) if default_variant else None,
                     "algorithmic_bytes": b_gat, "avg_launch_us": round(ms_gather * 1e3, 2)},
        "roofline_append": {"bound": "hbm", "kernel": "quantize_append_kernel",
                            "achieved": round(gbps(b_app, ms_append), 1), "peak": HBM_PEAK_GBPS,
                            "unit": "GB/s", "frac": round(gbps(b_app, ms_append) / HBM_PEAK_GBPS, 4),
                            "frac_of_probe": round(gbps(b_app, ms_append) / probe_append, 4),
                            "traffic": measured_traffic("quantize_append_kernel", w.name) if default_variant else None,
                            "algorithmic_bytes": b_app, "avg_launch_us": round(ms_append * 1e3, 2)},
    }

    if path == oqm.TOM_SCORE_TOKEN_GEMM:
        # the per-token contraction runs on the float64 matrix cores: 2 * T_q * H_k*d flop per group
        flop = 2.0 * w.t_q * w.n_kv_heads * w.head_dim * T * L
        out["roofline_score"] = {"bound": "mfma", "kernel": "score_token_gemm_kernel (+ query fold)",
                                 "achieved": round(flop / (ms_score * 1e-3) / 1e12, 2), "peak": 78.6,
                                 "unit": "TFLOP/s", "frac": round(flop / (ms_score * 1e-3) / 1e12 / 78.6, 4),
                                 "traffic": measured_traffic("score_token_gemm_kernel", w.name) if default_variant else None,
                                 "flop": flop, "avg_launch_us": round(ms_score * 1e3, 2)}
    if not args.no_cpu_baseline:
        nb = max(1, args.cpu_sample_batches if fpa > 1 else 64)
        host = [(k.cpu(), v.cpu()) for k, v in batches[:min(nb, n_batches)]]
        sample = [host[i % len(host)] for i in range(nb)]      # cycle the resident batches
        threads = min(16, os.cpu_count() or 1)
        out["cpu_baseline"] = cpu_baseline(w, sample, queries[0].cpu(), threads, 1 if tok else 0, args.bits, args.meta)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 3)
        out["cpu_baseline"]["one_core"]["value"] = round(out["cpu_baseline"]["one_core"]["value"], 3)
    print(json.dumps(out))
    mem.close()


if __name__ == "__main__":
    main()
