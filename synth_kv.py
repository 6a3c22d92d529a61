"""Seeded synthetic K/V streams and queries shaped like a LLaVA-OV-7B (Qwen2-7B
backbone: 28 layers, 4 KV heads, 28 query heads, head_dim 128) video stream.

This module only draws random tensors.  It holds none of the method's
arithmetic and is the one piece of code that both the CPU oracle's tests and
the GPU path's tests/bench use, so that the two sides see the same bits.

The five workloads below are the benchmark configurations; they stand in for
the post-LLM K/V of real video frames (no dataset or weights are used).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    group_tokens: int      # G: tokens per frame-group (one frame per group)
    n_frames: int          # T: frame-groups in the stream
    qgroup: int            # gs: quant-group size along head_dim
    t_q: int               # query tokens
    top_k: int             # frame-groups retrieved per layer
    dtype: str             # "f32" | "bf16" | "f16"
    sim: str               # "dot" | "cosine"
    seed: int
    kind: str              # value recipe: "normal" | "layer_std" | "outlier"
    frames_per_append: int  # frames handed to one quantize-append call


WORKLOADS = {
    # tiny CPU-checkable stream
    "C1": Workload("C1", 1, 2, 2, 64, 16, 32, 32, 1, 4, "f32", "dot", 1, "normal", 32),
    # one Qwen2-7B-shaped layer
    "C2": Workload("C2", 1, 4, 28, 128, 196, 256, 64, 16, 32, "bf16", "cosine", 2, "normal", 256),
    # all 28 layers, per-layer std in [0.5, 2]
    "C3": Workload("C3", 28, 4, 28, 128, 196, 1024, 64, 32, 64, "bf16", "cosine", 3, "layer_std", 32),
    # hour-long 1 fps stream, one frame per append, 100 interleaved queries
    "C4": Workload("C4", 28, 4, 28, 128, 196, 3600, 64, 32, 64, "bf16", "cosine", 4, "layer_std", 1),
    # outlier-heavy keys, gs 32, 64-token query (dense score contraction)
    "C5": Workload("C5", 28, 4, 28, 128, 196, 1024, 32, 64, 128, "bf16", "cosine", 5, "outlier", 32),
    # the stream of the paper's latency breakdown (Fig. 5): 64 frames of 50 kept tokens, FP16,
    # stored 8 frames at a time (the encoder batch), all 64 groups within the 12k-token budget
    "P64": Workload("P64", 28, 4, 28, 128, 50, 64, 64, 32, 64, "f16", "cosine", 6, "layer_std", 8),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller/larger variant of a workload (same recipe, different sizes)."""
    return replace(w, **kw)


_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def torch_dtype(w: Workload) -> torch.dtype:
    return _TORCH_DTYPE[w.dtype]


def _gen(device, *seed_parts: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for p in seed_parts:
        s = (s * 6364136223846793005 + 1442695040888963407 + int(p)) % (1 << 63)
    g.manual_seed(s)
    return g


def layer_std(w: Workload, device="cpu") -> torch.Tensor:
    """Per-layer standard deviation, uniform in [0.5, 2] ("layer_std"/"outlier": seeded)."""
    if w.kind == "normal":
        return torch.ones(w.n_layers, device=device)
    g = _gen("cpu", w.seed, 101)
    return (0.5 + 1.5 * torch.rand(w.n_layers, generator=g)).to(device)


def outlier_gain(w: Workload, device="cpu") -> torch.Tensor:
    """[L][H_k][d] multiplier: 20 on 4 channel ids drawn once per (layer, head), else 1."""
    g = _gen("cpu", w.seed, 202)
    a = torch.ones(w.n_layers, w.n_kv_heads, w.head_dim)
    for l in range(w.n_layers):
        for h in range(w.n_kv_heads):
            ids = torch.randperm(w.head_dim, generator=g)[:4]
            a[l, h, ids] = 20.0
    return a.to(device)


def kv_frames(w: Workload, frame0: int, n_frames: int, device="cpu"):
    """K, V of frames [frame0, frame0 + n_frames): two tensors [F][L][H_k][G][d] in the
    workload's dtype, drawn from a generator seeded by (workload seed, frame0, n_frames)
    on `device` (so a given call is reproducible; CPU and GPU draws differ)."""
    dev = torch.device(device)
    g = _gen(dev.type if dev.type == "cpu" else dev, w.seed, 7, frame0, n_frames)
    shape = (n_frames, w.n_layers, w.n_kv_heads, w.group_tokens, w.head_dim)
    k = torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
    v = torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
    if w.kind == "layer_std":
        sd = layer_std(w, dev).view(1, -1, 1, 1, 1)
        k *= sd
        v *= sd
    elif w.kind == "outlier":
        # K = gain * normal + Student-t(3) noise; V stays N(0, 1)
        z = torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
        chi = torch.zeros(shape, device=dev, dtype=torch.float32)
        for _ in range(3):
            chi += torch.randn(shape, generator=g, device=dev, dtype=torch.float32) ** 2
        k = k * outlier_gain(w, dev).view(1, w.n_layers, w.n_kv_heads, 1, w.head_dim) \
            + z / torch.sqrt(chi / 3.0)
    dt = torch_dtype(w)
    return k.to(dt).contiguous(), v.to(dt).contiguous()


def query(w: Workload, query_id: int = 0, device="cpu") -> torch.Tensor:
    """Q [L][H_q][T_q][d] ~ N(0, 1) in the workload's dtype."""
    dev = torch.device(device)
    g = _gen(dev.type if dev.type == "cpu" else dev, w.seed, 13, query_id)
    q = torch.randn((w.n_layers, w.n_q_heads, w.t_q, w.head_dim), generator=g, device=dev,
                    dtype=torch.float32)
    return q.to(torch_dtype(w)).contiguous()


def as_numpy_bits(t: torch.Tensor):
    """CPU numpy view of a tensor: float32 as is, bf16/f16 as their uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    return t.view(torch.int16).numpy().view("uint16")
