#!/usr/bin/env python3
"""Benchmark of the OQM hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
    quantize-append of `frames_per_append` frames (all layers, K and V)
    -> score all stored frame-groups against a T_q-token query
    -> top-k per layer -> dequant-gather of the k groups into the bf16 active KV buffer.
All inputs are resident in HBM before the timed region.  The store is pre-filled, and every
step overwrites a rotating window of group slots so that it always holds the full stream.

Without --workload the run is: the headline workload C3 (timed over --steps steps), then short
legs of C2, C5 and C4 (per-kernel figures only) and C4's live stream (3600 one-frame appends
with a query after every 36th), all reported in ONE JSON line (`workloads` holds the extra
legs).  With --workload X only that leg runs: the commands the profiles are taken with.
"""
from __future__ import annotations

import argparse
import ctypes as C
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
F64_MATRIX_PEAK_TFLOPS = 78.6   # MI355X published float64 matrix rate
METRIC = "OQM quantize-append + retrieve/dequant HBM GB/s (% of peak); retrieval ms/query"
EXTRA_LEGS = ("C2", "C5", "C4")


# ------------------------------------------------------------------ algorithmic bytes
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


# ------------------------------------------------------------------ committed counter summaries
def kernel_sources_hash():
    """SHA-256 over the kernels' sources (every .hip / .h under csrc/ except the benchmark-only
    probe and the division self-check), in name order: ties a committed counter summary to the
    code it was taken from."""
    d = os.path.join(ROOT, "paper_2510_18269_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")) and name not in ("bench_probe.hip", "selfcheck_division.hip"):
            h.update(name.encode() + b"\0")
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel, workload):
    """(HBM bytes per launch read + written, note).  The bytes come from the committed rocprofv3
    FETCH_SIZE / WRITE_SIZE summary of `bench.py --workload <workload>`; they are reported only
    if that summary names the kernel sources this run was built from, else None and why."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_bench_{workload.lower()}.txt")
    src = f"profiles/hbm_traffic_bench_{workload.lower()}.txt"
    try:
        with open(path) as f:
            lines = f.read().splitlines()
    except OSError:
        return None, f"no committed counter summary ({src})"
    stamped = [l.split()[1] for l in lines if l.startswith("kernel_sources_sha256 ") and len(l.split()) == 2]
    if not stamped:
        return None, f"{src} does not say which kernel sources it was taken from"
    if stamped[0] != kernel_sources_hash():
        return None, f"{src} was taken from other kernel sources (sha256 {stamped[0][:12]}...): re-profile"
    for line in lines:
        p = line.split()
        if len(p) == 5 and p[0] == "traffic" and p[1] == kernel and p[2] == workload:
            return int(p[3]) + int(p[4]), f"rocprofv3 FETCH_SIZE + WRITE_SIZE, committed summary {src} of the same kernel sources"
    return None, f"{src} has no line for {kernel}"


def traced_duration_us(kernel, workload):
    """Average duration of `kernel` in the committed rocprofv3 kernel trace of
    `bench.py --workload <workload>` (another run of the same kernel sources), or None."""
    path = os.path.join(ROOT, "profiles", f"kernel_trace_bench_{workload.lower()}.txt")
    try:
        with open(path) as f:
            lines = f.read().splitlines()
    except OSError:
        return None
    stamped = [l.split()[1] for l in lines if l.startswith("kernel_sources_sha256 ") and len(l.split()) == 2]
    if not stamped or stamped[0] != kernel_sources_hash():
        return None
    for line in lines:
        if line.startswith(kernel + "<") or line.startswith(kernel + " "):
            tail = line.rsplit(None, 5)      # name ... calls avg min max total
            try:
                return float(tail[2])
            except (IndexError, ValueError):
                return None
    return None


def load_probe_lib():
    """The benchmark-only shared object (stream probes); not part of the library."""
    path = os.path.join(ROOT, "paper_2510_18269_amd", "libtom_bench_probe.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build first (python -m paper_2510_18269_amd.build)")
    lib = C.CDLL(path)
    lib.bench_stream_probe.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.bench_stream_probe.restype = C.c_int
    lib.bench_event_create.argtypes = []
    lib.bench_event_create.restype = C.c_void_p
    lib.bench_event_record.argtypes = [C.c_void_p, C.c_void_p]
    lib.bench_event_record.restype = C.c_int
    lib.bench_event_elapsed_ms.argtypes = [C.c_void_p, C.c_void_p]
    lib.bench_event_elapsed_ms.restype = C.c_float
    lib.bench_event_destroy.argtypes = [C.c_void_p]
    lib.bench_event_destroy.restype = None
    return lib


class StreamEvent:
    """A HIP timing event recorded on torch's current stream (the stream every library call of
    this benchmark is queued on), created without the system-scope fence a default event
    carries: same interface as torch.cuda.Event, about half the cost to the stream."""
    lib = None
    torch = None

    def __init__(self):
        self.h = StreamEvent.lib.bench_event_create()
        assert self.h, "hipEventCreateWithFlags failed"

    def record(self):
        rc = StreamEvent.lib.bench_event_record(self.h, StreamEvent.torch.cuda.current_stream().cuda_stream)
        assert rc == 0, f"hipEventRecord: hipError {rc}"

    def elapsed_time(self, other):
        ms = StreamEvent.lib.bench_event_elapsed_ms(self.h, other.h)
        assert ms >= 0.0, "hipEventElapsedTime failed (events not complete?)"
        return ms

    def __del__(self):
        if self.h and StreamEvent.lib is not None:
            StreamEvent.lib.bench_event_destroy(self.h)
            self.h = None


# ------------------------------------------------------------------ the oracle on the host cores
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
    return {"value": round(total / dtm / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{w.name}: {F} frames x {L} layers appended ({len(kb)} calls) + 1 query "
                      f"(T_q={w.t_q}) scored over {F} groups, top-{k_eff} dequant-gathered; "
                      f"{ea + eg} K/V elements in {dtm:.2f} s",
            "one_core": {"value": round(total / L / dt1 / 1e9, 3), "unit": "GB/s",
                         "sample": f"layer 0 of the same sample again on one thread, {dt1:.2f} s; run after the "
                                   f"{threads}-thread pass, so its inputs and the store's layer-0 slice are "
                                   "already in the host caches / page tables"},
            "seconds": round(dtm, 3)}


# ------------------------------------------------------------------ one workload on the GPU
class Leg:
    """Sets up one workload on the GPU (store pre-filled, inputs resident) and times steps."""

    def __init__(self, name, args, torch, oqm, synth_kv, probe_lib):
        self.torch, self.oqm, self.synth_kv, self.probe_lib = torch, oqm, synth_kv, probe_lib
        self.args = args
        dev = self.dev = "cuda:0"
        w = synth_kv.WORKLOADS[name]
        qaxis = args.qaxis or ("tokens" if name == "P64" else "head_dim")
        if args.group_tokens:
            w = synth_kv.scaled(w, group_tokens=args.group_tokens)
        self.tok = tok = qaxis == "tokens"
        fpa = args.frames_per_append or (w.frames_per_append if w.frames_per_append > 1 else 1)
        self.fpa = fpa = min(fpa, w.n_frames)
        self.T = T = (w.n_frames // fpa) * fpa
        self.eb = eb = 4 if w.dtype == "f32" else 2
        dtc = {"f32": oqm.TOM_F32, "bf16": oqm.TOM_BF16, "f16": oqm.TOM_F16}[w.dtype]
        cfg = oqm.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens,
                              w.qgroup, T, qaxis=oqm.TOM_QAXIS_TOKENS if tok else oqm.TOM_QAXIS_HEAD_DIM,
                              bits=args.bits, in_dtype=dtc, out_dtype=dtc,
                              meta_dtype=oqm.TOM_BF16 if args.meta == "bf16" else oqm.TOM_F32,
                              sim=oqm.TOM_SIM_COSINE if w.sim == "cosine" else oqm.TOM_SIM_DOT)
        self.mem = mem = oqm.Memory.allocate(cfg, dev)
        self.w_gen = w          # what the inputs are drawn from
        if tok:   # byte model: one (scale, zero) pair per channel and tile instead of per gs elements
            w = synth_kv.scaled(w, qgroup=w.group_tokens)
        self.w = w
        self.L = L = w.n_layers
        self.meta_b = 4 if args.meta == "bf16" else 8
        # distinct input batches, more than the 256 MB last-level cache can hold, rotated per step
        batch_bytes = bytes_append(w, fpa, eb, args.bits, self.meta_b)[0]
        self.n_batches = max(2, min(T // fpa, int(3.0e9 // max(batch_bytes, 1)) or 1, 64))
        self.batches = [synth_kv.kv_frames(self.w_gen, i * fpa, fpa, dev) for i in range(self.n_batches)]
        self.queries = [synth_kv.query(self.w_gen, i, dev) for i in range(4)]
        self.path = oqm.TOM_SCORE_TOKEN_GEMM if name == "C5" else oqm.TOM_SCORE_MEAN_QUERY
        self.ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, w.t_q, self.path),
                              dtype=torch.uint8, device=dev)
        self.scores = torch.zeros((L, T), dtype=torch.float32, device=dev)
        self.idx = torch.zeros((L, w.top_k), dtype=torch.int32, device=dev)
        tdt = synth_kv.torch_dtype(w)
        shape = (L, w.n_kv_heads, w.top_k * w.group_tokens, w.head_dim)
        self.outs = [(torch.empty(shape, dtype=tdt, device=dev), torch.empty(shape, dtype=tdt, device=dev))
                     for _ in range(2)]
        self.k_eff = min(w.top_k, T)
        for i in range(T // fpa):      # pre-fill the whole store (untimed)
            k, v = self.batches[i % self.n_batches]
            oqm.tom_oqm_quantize_append(mem.handle, 0, L, fpa, k, v)
        torch.cuda.synchronize()
        assert mem.n_groups == T
        self.n_windows = T // fpa

    def close(self):
        self.mem.close()
        for a in ("batches", "queries", "ws", "scores", "idx", "outs", "mem"):
            setattr(self, a, None)
        self.torch.cuda.empty_cache()

    def step(self, i, ev=None):
        """One pass of the hot path.  Plain steps queue two library calls (append, then the
        one-call retrieval = score + top-k + gather back to back); an event step takes the same
        kernels through the separate calls with a HIP event after each, which is where the
        per-kernel durations come from (an event between two kernels costs the stream about
        5 us, so it is not paid on every step)."""
        oqm, mem, w, L, T, fpa = self.oqm, self.mem, self.w, self.L, self.T, self.fpa
        k, v = self.batches[i % self.n_batches]
        oqm.tom_oqm_set_num_groups(mem.handle, (i % self.n_windows) * fpa)
        if ev:
            ev[0].record()
        oqm.tom_oqm_quantize_append(mem.handle, 0, L, fpa, k, v)
        if ev:
            ev[1].record()
        oqm.tom_oqm_set_num_groups(mem.handle, T)
        q = self.queries[i % len(self.queries)]
        ko, vo = self.outs[i % 2]
        if not ev:
            oqm.tom_oqm_retrieve(mem.handle, 0, L, q, w.t_q, w.top_k, self.scores, T, self.idx, ko, vo, self.ws,
                                 path=self.path)
            return
        oqm.tom_oqm_score_groups(mem.handle, 0, L, q, w.t_q, self.scores, T, None, self.path, self.ws)
        ev[2].record()
        oqm.tom_oqm_topk(self.scores, T, L, T, w.top_k, self.idx)
        ev[3].record()
        oqm.tom_oqm_dequant_gather(mem.handle, 0, L, self.idx, w.top_k, self.k_eff, ko, vo)
        ev[4].record()

    def run(self, steps, warmup, probes, default_variant):
        torch, w, L, T, fpa, eb = self.torch, self.w, self.L, self.T, self.fpa, self.eb
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        # eight steps, evenly spread, carry per-kernel events, whatever --steps is (all of them below 8)
        n_ev = min(steps, 8)
        ev_steps = {(j * steps) // n_ev for j in range(n_ev)}
        events = [[StreamEvent() for _ in range(5)] if i in ev_steps else None
                  for i in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i, events[i])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        events = [e for e in events if e]

        # latency of the one-call retrieval alone: 20 queries back to back between two events
        rev = [StreamEvent() for _ in range(2)]
        rev[0].record()
        for i in range(20):
            ko, vo = self.outs[i % 2]
            self.oqm.tom_oqm_retrieve(self.mem.handle, 0, L, self.queries[i % len(self.queries)], w.t_q, w.top_k,
                                      self.scores, T, self.idx, ko, vo, self.ws, path=self.path)
        rev[1].record()
        torch.cuda.synchronize()
        ms_retrieve_call = rev[0].elapsed_time(rev[1]) / 20

        # what an empty interval between two events reads: an upper bound of the events' own cost,
        # which every per-kernel figure below includes (it matters for the short kernels)
        oev = [StreamEvent() for _ in range(21)]
        for e in oev:
            e.record()
        torch.cuda.synchronize()
        event_overhead_us = sum(oev[i].elapsed_time(oev[i + 1]) for i in range(20)) / 20 * 1e3

        def avg_ms(a, b):
            return sum(e[a].elapsed_time(e[b]) for e in events) / len(events)

        ms_append, ms_score, ms_topk, ms_gather = avg_ms(0, 1), avg_ms(1, 2), avg_ms(2, 3), avg_ms(3, 4)
        ms_step = wall * 1e3 / steps
        a = self.args
        b_app, _ = bytes_append(w, fpa, eb, a.bits, self.meta_b)
        b_gat, _ = bytes_gather(w, self.k_eff, eb, a.bits, self.meta_b)
        b_sc, b_tk = bytes_score(w, T, eb), bytes_topk(w, T, self.k_eff)
        total_bytes = b_app + b_gat + b_sc + b_tk
        gbps = lambda b, ms: b / (ms * 1e-3) / 1e9

        def roof(kernel, b, ms, probe):
            traffic, note = measured_traffic(kernel, w.name) if default_variant else (None, "not the default variant")
            traced = traced_duration_us(kernel, w.name) if default_variant else None
            return {"bound": "hbm", "kernel": kernel, "achieved": round(gbps(b, ms), 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(gbps(b, ms) / HBM_PEAK_GBPS, 4),
                    "frac_of_probe": round(gbps(b, ms) / probe, 4) if probe else None,
                    "traffic": traffic, "traffic_source": note,
                    "algorithmic_bytes": b, "avg_launch_us": round(ms * 1e3, 2), "launches_timed": len(events),
                    # context: the same kernel in the committed rocprofv3 kernel trace (another run, same
                    # sources); the event interval above is this plus the events' own cost
                    "committed_kernel_trace_us": traced,
                    "frac_by_committed_kernel_trace": round(b / (traced * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if traced else None}

        tok = self.tok
        r = {
            "workload": f"{w.name}: {L} layers, {w.n_kv_heads} KV heads ({w.n_q_heads} query heads), "
                        f"head_dim {w.head_dim}, {w.dtype} K/V, {T} frames x {w.group_tokens} tokens stored, "
                        f"{fpa} frames per quantize-append, {a.bits}-bit codes, {a.meta} scale/zero, "
                        + (f"scale/zero per channel over the {w.group_tokens} tokens, " if tok else
                           f"quant-group {w.qgroup} over head_dim, ") +
                        f"{w.t_q}-token query, top-{self.k_eff} groups dequant-gathered to {w.dtype}",
            "value_recipe": w.kind, "io_dtype": w.dtype,
            "score_path": "token_gemm" if self.path == self.oqm.TOM_SCORE_TOKEN_GEMM else "mean_query",
            "input_batches_rotated": self.n_batches, "steps": steps, "steps_with_kernel_events": len(events),
            "ms_per_step": round(ms_step, 4), "GBps": round(gbps(total_bytes, ms_step), 1),
            "pct_of_hbm_peak": round(100 * gbps(total_bytes, ms_step) / HBM_PEAK_GBPS, 2),
            "bytes_per_step": total_bytes,
            "append": {"ms": round(ms_append, 4), "GBps": round(gbps(b_app, ms_append), 1),
                       "pct_of_peak": round(100 * gbps(b_app, ms_append) / HBM_PEAK_GBPS, 2),
                       "tokens_per_s": round(fpa * w.group_tokens / (ms_append * 1e-3), 1), "bytes": b_app},
            "score": {"ms": round(ms_score, 4), "GBps": round(gbps(b_sc, ms_score), 1), "bytes": b_sc},
            "topk": {"ms": round(ms_topk, 4)},
            "gather": {"ms": round(ms_gather, 4), "GBps": round(gbps(b_gat, ms_gather), 1),
                       "pct_of_peak": round(100 * gbps(b_gat, ms_gather) / HBM_PEAK_GBPS, 2), "bytes": b_gat},
            "event_overhead_us": round(event_overhead_us, 2),
            "retrieval_ms_per_query": round(ms_retrieve_call, 4),
            "retrieval_ms_per_query_separate_calls": round(ms_score + ms_topk + ms_gather, 4),
            "roofline": roof("dequant_gather_kernel", b_gat, ms_gather, probes.get("gather")),
            "roofline_append": roof("quantize_append_tokens_kernel" if tok else "quantize_append_kernel", b_app,
                                    ms_append, probes.get("append")),
        }
        if self.path == self.oqm.TOM_SCORE_TOKEN_GEMM:
            # the per-token contraction runs on the float64 matrix cores: 2 * T_q * H_k*d flop per group
            flop = 2.0 * w.t_q * w.n_kv_heads * w.head_dim * T * L
            traffic, note = measured_traffic("score_token_gemm_kernel", w.name) if default_variant else (None, "not the default variant")
            r["roofline_score"] = {"bound": "mfma", "kernel": "score_token_gemm_kernel (+ query fold)",
                                   "achieved": round(flop / (ms_score * 1e-3) / 1e12, 2),
                                   "peak": F64_MATRIX_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": round(flop / (ms_score * 1e-3) / 1e12 / F64_MATRIX_PEAK_TFLOPS, 4),
                                   "traffic": traffic, "traffic_source": note,
                                   "flop": flop, "avg_launch_us": round(ms_score * 1e3, 2),
                                   "launches_timed": len(events)}
        return r


def c4_live_stream(torch, oqm, synth_kv, args):
    """Configuration 4 as a live stream: 3600 one-frame appends, and after every 36th frame one
    query (T_q = 32, top-64) over what has been stored so far, so the score step sees
    T = 36, 72, ..., 3600 (the supplement's streaming protocol: a question is answered from the
    frames that arrived before it).  Per-query latency is taken with a HIP event pair around each
    one-call retrieval, per-append time from an event pair around each block of 36 appends."""
    dev = "cuda:0"
    w = synth_kv.WORKLOADS["C4"]
    L, T, every = w.n_layers, w.n_frames, 36
    cfg = oqm.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens, w.qgroup, T,
                          in_dtype=oqm.TOM_BF16, out_dtype=oqm.TOM_BF16, sim=oqm.TOM_SIM_COSINE)
    mem = oqm.Memory.allocate(cfg, dev)
    frames = [synth_kv.kv_frames(w, i, 1, dev) for i in range(64)]      # 64 distinct frames, rotated
    queries = [synth_kv.query(w, i, dev) for i in range(4)]
    ws = torch.empty(oqm.tom_oqm_score_workspace_bytes(mem.handle, L, w.t_q, oqm.TOM_SCORE_MEAN_QUERY),
                     dtype=torch.uint8, device=dev)
    scores = torch.zeros((L, T), dtype=torch.float32, device=dev)
    idx = torch.zeros((L, w.top_k), dtype=torch.int32, device=dev)
    tdt = synth_kv.torch_dtype(w)
    shape = (L, w.n_kv_heads, w.top_k * w.group_tokens, w.head_dim)
    outs = [(torch.empty(shape, dtype=tdt, device=dev), torch.empty(shape, dtype=tdt, device=dev)) for _ in range(2)]
    for f in range(72):                # warm-up: two blocks and two queries, then start over
        oqm.tom_oqm_quantize_append(mem.handle, 0, L, 1, *frames[f % 64])
        if (f + 1) % every == 0:
            oqm.tom_oqm_retrieve(mem.handle, 0, L, queries[0], w.t_q, w.top_k, scores, T, idx, *outs[0], ws,
                                 path=oqm.TOM_SCORE_MEAN_QUERY)
    torch.cuda.synchronize()
    oqm.tom_oqm_reset(mem.handle)
    n_q = T // every
    ev = [[StreamEvent() for _ in range(3)] for _ in range(n_q)]
    t0 = time.perf_counter()
    for j in range(n_q):
        ev[j][0].record()
        for f in range(j * every, (j + 1) * every):
            oqm.tom_oqm_quantize_append(mem.handle, 0, L, 1, *frames[f % 64])
        ev[j][1].record()
        oqm.tom_oqm_retrieve(mem.handle, 0, L, queries[j % 4], w.t_q, w.top_k, scores, T, idx, *outs[j % 2], ws,
                             path=oqm.TOM_SCORE_MEAN_QUERY)
        ev[j][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert mem.n_groups == T
    app = sorted(e[0].elapsed_time(e[1]) / every * 1e3 for e in ev)       # us per one-frame append
    ret = [e[1].elapsed_time(e[2]) for e in ev]                            # ms per query, in stream order
    rs = sorted(ret)
    pct = lambda s, p: s[min(len(s) - 1, int(round(p * (len(s) - 1))))]
    eb = 2
    b_app = bytes_append(w, 1, eb)[0]
    out = {"what": f"{T} one-frame quantize-appends (28 layers), one {w.t_q}-token query after every {every}th frame "
                   f"over the T = {every} ... {T} groups stored so far, top-{w.top_k} (all of them while T < {w.top_k}) "
                   "dequant-gathered",
           "frames": T, "queries": n_q, "stream_wall_ms": round(wall * 1e3, 2),
           "append_us_per_frame": {"mean": round(sum(app) / len(app), 2), "p50": round(pct(app, 0.5), 2),
                                   "p99": round(pct(app, 0.99), 2),
                                   "what": "HIP event pair around each block of 36 back-to-back calls, / 36"},
           "append_GBps": round(b_app / (sum(app) / len(app) * 1e-6) / 1e9, 1),
           "retrieval_ms_per_query": {"mean": round(sum(ret) / len(ret), 4), "p50": round(pct(rs, 0.5), 4),
                                      "p99": round(pct(rs, 0.99), 4), "min": round(rs[0], 4), "max": round(rs[-1], 4),
                                      "first_T36": round(ret[0], 4), "last_T3600": round(ret[-1], 4),
                                      "what": "HIP event pair around each one-call retrieval (includes about one "
                                              "empty event interval)"}}
    mem.close()
    del frames, outs, scores, ws
    torch.cuda.empty_cache()
    return out


def run_probes(torch, probe_lib):
    """What the machine reaches for the byte mix of the two big kernels: arithmetic-free linear
    streams over rotating regions far larger than the last-level cache.  Depth 1 = one item per
    thread; depth 4 = four pieces per workgroup, loads first (the fastest form found)."""
    dev = "cuda:0"

    def probe(mode, depth, read_b, write_b):
        items = 44 << 20
        n_src, n_dst = (12, 4) if read_b < write_b else (4, 12)
        src = torch.empty(items * read_b * n_src, dtype=torch.uint8, device=dev).random_()
        dst = torch.empty(items * write_b * n_dst, dtype=torch.uint8, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = 12
        for i in range(3 + reps):
            if i == 3:
                ev[0].record()
            rc = probe_lib.bench_stream_probe(mode, depth, src.data_ptr() + (i % n_src) * items * read_b,
                                              dst.data_ptr() + (i % n_dst) * items * write_b, items,
                                              torch.cuda.current_stream().cuda_stream)
            assert rc == 0, f"stream probe: hipError {rc}"
        ev[1].record()
        torch.cuda.synchronize()
        g = reps * items * (read_b + write_b) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
        del src, dst
        return g

    # a plain device-to-device copy of known size (1 GiB read + 1 GiB written): the reference the
    # HBM byte counters are calibrated with
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
    g1, g4 = probe(0, 1, 4, 16), probe(0, 4, 4, 16)
    a1, a4 = probe(1, 1, 16, 4), probe(1, 4, 16, 4)
    torch.cuda.empty_cache()
    return {"gather": max(g1, g4), "append": max(a1, a4),
            "report": {"gather_mix_GBps": round(max(g1, g4), 1), "append_mix_GBps": round(max(a1, a4), 1),
                       "gather_mix_depth1_GBps": round(g1, 1), "gather_mix_depth4_GBps": round(g4, 1),
                       "append_mix_depth1_GBps": round(a1, 1), "append_mix_depth4_GBps": round(a4, 1),
                       "torch_copy_GBps": round(copy_gbps, 1),
                       "what": "arithmetic-free linear streams with the kernels' read/write mix (4 B in / 16 B "
                               "out, 16 B in / 4 B out), same run; depth = 1 KB / 4 KB pieces per workgroup with "
                               "all loads issued before the stores; frac_of_probe is against the faster depth"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, choices=["C2", "C3", "C4", "C5", "P64"],
                    help="run this workload alone (default: C3 as the headline, then short legs of C2, C5, C4 "
                         "and C4's live stream); P64 = the 64-frame stream of the paper's latency breakdown")
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
    ap.add_argument("--extra-steps", type=int, default=20, help="timed steps of each extra leg")
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
    probe_lib = load_probe_lib()
    StreamEvent.lib, StreamEvent.torch = probe_lib, torch
    probes = run_probes(torch, probe_lib)
    default_variant = (args.qaxis in (None, "head_dim") and args.bits == 4 and not args.group_tokens
                       and not args.frames_per_append and args.meta == "f32")
    head_name = args.workload or "C3"
    if head_name == "P64" and args.qaxis in (None, "tokens"):
        default_variant = False

    leg = Leg(head_name, args, torch, oqm, synth_kv, probe_lib)
    r = leg.run(args.steps, args.warmup, probes, default_variant)
    out = {
        "metric": METRIC, "value": r["GBps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": r["workload"], "value_recipe": r["value_recipe"], "io_dtype": r["io_dtype"],
                   "arithmetic": "float32 scale / zero / code arithmetic, float64 key sums and scores, "
                                 f"{r['io_dtype']} K/V in and out",
                   "score_path": r["score_path"], "input_batches_rotated": r["input_batches_rotated"],
                   "steps_with_kernel_events": r["steps_with_kernel_events"]},
        "pct_of_hbm_peak": r["pct_of_hbm_peak"], "copy_GBps": probes["report"]["torch_copy_GBps"],
        "probe": probes["report"], "bytes_per_step": r["bytes_per_step"],
    }
    for key in ("append", "score", "topk", "gather", "event_overhead_us", "retrieval_ms_per_query",
                "retrieval_ms_per_query_separate_calls", "roofline", "roofline_append", "roofline_score"):
        if key in r:
            out[key] = r[key]
    host = None
    if not args.no_cpu_baseline:
        nb = max(1, args.cpu_sample_batches if leg.fpa > 1 else 64)
        host = [(k.cpu(), v.cpu()) for k, v in leg.batches[:min(nb, leg.n_batches)]]
        host = ([host[i % len(host)] for i in range(nb)], leg.queries[0].cpu(), leg.w)     # cycle the resident batches
    leg.close()

    if args.workload is None:
        # the other configurations: short legs for their per-kernel figures, and C4's live stream
        extra = {}
        for name in EXTRA_LEGS:
            x = Leg(name, args, torch, oqm, synth_kv, probe_lib)
            e = x.run(args.extra_steps, 3, probes, default_variant)
            x.close()
            extra[name] = {k: e[k] for k in ("workload", "steps", "steps_with_kernel_events", "ms_per_step", "GBps",
                                             "append", "score", "topk", "gather", "retrieval_ms_per_query",
                                             "roofline", "roofline_append", "roofline_score") if k in e}
        extra["C4"]["live_stream"] = c4_live_stream(torch, oqm, synth_kv, args)
        out["workloads"] = extra

    if host is not None:
        threads = min(16, os.cpu_count() or 1)
        out["cpu_baseline"] = cpu_baseline(host[2], host[0], host[1], threads, 1 if leg.tok else 0, args.bits, args.meta)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
