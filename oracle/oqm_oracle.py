"""ctypes front end of the CPU oracle (oracle/oqm_oracle.c).

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this module.  It holds no arithmetic of the
method: every number comes out of the C file, this file only marshals numpy
arrays.  bf16 / f16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oqm_oracle.c")
_LIB = os.path.join(_HERE, "liboqm_oracle.so")

F32, BF16, F16 = 0, 1, 2
QAXIS_HEAD_DIM, QAXIS_TOKENS = 0, 1
SIM_DOT, SIM_COSINE = 0, 1
ORDER_INDEX_ASC, ORDER_SCORE_DESC = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_kv_heads", "n_q_heads", "head_dim", "group_tokens", "qgroup",
        "qaxis", "bits", "capacity_groups", "in_dtype", "out_dtype", "sim", "meta_dtype")]


@dataclass
class Store:
    """Host-side OQM memory, in the layout the oracle's header comment states."""
    cfg: Config
    codes: np.ndarray   # uint8
    scale: np.ndarray   # float32
    zero: np.ndarray    # float32
    keys: np.ndarray    # float32 [L][T_cap][H_k][d]
    n_groups: int = 0


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, i32, i64, f32p = C.c_void_p, C.c_int32, C.c_int64, C.c_void_p
        L.tomref_to_f32.argtypes = [vp, i32, i64, f32p]
        L.tomref_to_f32.restype = None
        L.tomref_from_f32.argtypes = [f32p, i32, i64, vp]
        L.tomref_from_f32.restype = None
        L.tomref_kv_cache_bytes.argtypes = [i32, i32, i32, i32, i32, i64]
        L.tomref_kv_cache_bytes.restype = C.c_double
        L.tomref_compression_ratio.argtypes = [i32, i32, i32]
        L.tomref_compression_ratio.restype = C.c_double
        L.tomref_bits_per_element.argtypes = [i32, i32, i32, i32]
        L.tomref_bits_per_element.restype = C.c_double
        L.tomref_k_from_budget.argtypes = [i64, i32, i64]
        L.tomref_k_from_budget.restype = i32
        L.tomref_meta_per_tile.argtypes = [i32, i32, i32, i32]
        L.tomref_meta_per_tile.restype = i64
        L.tomref_code_bytes_per_tile.argtypes = [i32, i32, i32]
        L.tomref_code_bytes_per_tile.restype = i64
        L.tomref_quantize_tile.argtypes = [f32p, i32, i32, i32, i32, i32, i32, vp, vp, f32p, f32p]
        L.tomref_quantize_tile.restype = i32
        L.tomref_dequant_tile.argtypes = [vp, f32p, f32p, i32, i32, i32, i32, i32, f32p]
        L.tomref_dequant_tile.restype = i32
        L.tomref_summary_key.argtypes = [f32p, i32, i32, f32p]
        L.tomref_summary_key.restype = None
        L.tomref_quantize_append.argtypes = [C.POINTER(Config), vp, f32p, f32p, f32p, i32, i32,
                                             i32, i32, vp, vp, vp, C.POINTER(C.c_int64)]
        L.tomref_quantize_append.restype = i32
        L.tomref_score_groups.argtypes = [C.POINTER(Config), f32p, i32, i32, i32, vp, i32, i32,
                                          f32p, i64, f32p]
        L.tomref_score_groups.restype = i32
        L.tomref_topk.argtypes = [f32p, i64, i32, i32, i32, i32, vp]
        L.tomref_topk.restype = i32
        L.tomref_dequant_gather.argtypes = [C.POINTER(Config), vp, f32p, f32p, i32, i32, i32,
                                            vp, i32, i32, vp, vp]
        L.tomref_dequant_gather.restype = i32
        L.tomref_assemble_active.argtypes = [C.POINTER(Config), vp, f32p, f32p, i32, i32, i32,
                                             vp, i32, i32, i32, vp, vp, vp, vp]
        L.tomref_assemble_active.restype = i32
        _lib = L
    return _lib


def _p(a: np.ndarray | None):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle wrapper takes contiguous arrays"
    return a.ctypes.data_as(C.c_void_p)


def _np_dtype(dtype: int):
    return np.float32 if dtype == F32 else np.uint16


# ---------------------------------------------------------------- conversions
def to_f32(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=_np_dtype(dtype))
    out = np.empty(a.shape, np.float32)
    lib().tomref_to_f32(_p(a), dtype, a.size, _p(out))
    return out


def from_f32(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, _np_dtype(dtype))
    lib().tomref_from_f32(_p(a), dtype, a.size, _p(out))
    return out


# ---------------------------------------------------------------- closed forms
def kv_cache_bytes(L, N, H_kv, d_h, elem_bytes, frames) -> float:
    return lib().tomref_kv_cache_bytes(L, N, H_kv, d_h, elem_bytes, frames)


def compression_ratio(N, G, bits=4) -> float:
    return lib().tomref_compression_ratio(N, G, bits)


def bits_per_element(bits, qaxis, gs, G) -> float:
    return lib().tomref_bits_per_element(bits, qaxis, gs, G)


def k_from_budget(budget_tokens, G, stored_tokens) -> int:
    return lib().tomref_k_from_budget(budget_tokens, G, stored_tokens)


# ---------------------------------------------------------------- tile level
def quantize_tile(x: np.ndarray, gs: int, qaxis: int = QAXIS_HEAD_DIM, bits: int = 4,
                  meta_dtype: int = F32):
    """x: float32 [G][d] -> (unpacked [G][d] u8, packed [G][d*bits/8] u8, scale, zero)."""
    x = np.ascontiguousarray(x, np.float32)
    G, d = x.shape
    nm = lib().tomref_meta_per_tile(G, d, gs, qaxis)
    unpacked = np.empty((G, d), np.uint8)
    packed = np.empty((G, d * bits // 8), np.uint8)
    scale = np.empty(nm, np.float32)
    zero = np.empty(nm, np.float32)
    rc = lib().tomref_quantize_tile(_p(x), G, d, gs, qaxis, bits, meta_dtype, _p(unpacked), _p(packed),
                                    _p(scale), _p(zero))
    if rc != 0:
        raise ValueError("tomref_quantize_tile: bad shape")
    shape = (G, d // gs) if qaxis == QAXIS_HEAD_DIM else (d,)
    return unpacked, packed, scale.reshape(shape), zero.reshape(shape)


def dequant_tile(packed, scale, zero, G, d, gs, qaxis=QAXIS_HEAD_DIM, bits=4) -> np.ndarray:
    packed = np.ascontiguousarray(packed, np.uint8)
    scale = np.ascontiguousarray(scale, np.float32)
    zero = np.ascontiguousarray(zero, np.float32)
    out = np.empty((G, d), np.float32)
    rc = lib().tomref_dequant_tile(_p(packed), _p(scale), _p(zero), G, d, gs, qaxis, bits, _p(out))
    if rc != 0:
        raise ValueError("tomref_dequant_tile: bad shape")
    return out


def summary_key(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32)
    G, d = x.shape
    key = np.empty(d, np.float32)
    lib().tomref_summary_key(_p(x), G, d, _p(key))
    return key


# ---------------------------------------------------------------- the four calls
def make_config(n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup,
                capacity_groups, qaxis=QAXIS_HEAD_DIM, bits=4, in_dtype=BF16, out_dtype=BF16,
                sim=SIM_COSINE, meta_dtype=F32) -> Config:
    return Config(n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup, qaxis, bits,
                  capacity_groups, in_dtype, out_dtype, sim, meta_dtype)


def new_store(cfg: Config) -> Store:
    tiles = cfg.n_layers * 2 * cfg.capacity_groups * cfg.n_kv_heads
    cb = lib().tomref_code_bytes_per_tile(cfg.group_tokens, cfg.head_dim, cfg.bits)
    mt = lib().tomref_meta_per_tile(cfg.group_tokens, cfg.head_dim, cfg.qgroup, cfg.qaxis)
    return Store(cfg,
                 np.zeros(tiles * cb, np.uint8),
                 np.zeros(tiles * mt, np.float32),
                 np.zeros(tiles * mt, np.float32),
                 np.zeros((cfg.n_layers, cfg.capacity_groups, cfg.n_kv_heads, cfg.head_dim),
                          np.float32))


def quantize_append(st: Store, k: np.ndarray, v: np.ndarray, k_for_summary=None,
                    layer0: int = 0, strides=None, n_frames=None, n_layers=None,
                    commit: bool = True) -> int:
    """k, v: [F][n_layers][H_k][G][d] arrays in cfg.in_dtype (uint16 bits for bf16/f16),
    or any buffer when `strides` (frame, layer, head, token; in elements) is given."""
    cfg = st.cfg
    if strides is None:
        assert k.ndim == 5 and k.shape == v.shape
        F, nl, H, G, d = k.shape
        assert (H, G, d) == (cfg.n_kv_heads, cfg.group_tokens, cfg.head_dim)
        strides = (nl * H * G * d, H * G * d, G * d, d)
        n_frames, n_layers = F, nl
    sarr = (C.c_int64 * 4)(*strides)
    rc = lib().tomref_quantize_append(C.byref(cfg), _p(st.codes), _p(st.scale), _p(st.zero),
                                      _p(st.keys), st.n_groups, layer0, n_layers, n_frames,
                                      _p(k), _p(v), _p(k_for_summary), sarr)
    if rc != 0:
        raise ValueError(f"tomref_quantize_append failed rc={rc}")
    first = st.n_groups
    if commit:
        st.n_groups += n_frames
    return first


def score_groups(st: Store, q: np.ndarray, q_dtype: int, layer0: int = 0, n_layers=None,
                 want_token_scores: bool = False, n_groups=None):
    """q: [n_layers][H_q][T_q][d].  Returns scores [n_layers][n_groups] (and token scores)."""
    cfg = st.cfg
    q = np.ascontiguousarray(q)
    nl, Hq, tq, d = q.shape
    if n_layers is None:
        n_layers = nl
    T = st.n_groups if n_groups is None else n_groups
    scores = np.zeros((n_layers, max(T, 1)), np.float32)
    tok = np.zeros((n_layers, tq, T), np.float32) if want_token_scores else None
    rc = lib().tomref_score_groups(C.byref(cfg), _p(st.keys), T, layer0, n_layers, _p(q),
                                   q_dtype, tq, _p(scores), scores.shape[1], _p(tok))
    if rc != 0:
        raise ValueError(f"tomref_score_groups failed rc={rc}")
    scores = scores[:, :T]
    return (scores, tok) if want_token_scores else scores


def topk(scores: np.ndarray, k: int, order: int = ORDER_INDEX_ASC, n_groups=None):
    """scores: [rows][stride] float32.  Returns (idx [rows][k] int32, k_eff); entries
    beyond k_eff are -1."""
    scores = np.ascontiguousarray(scores, np.float32)
    rows, stride = scores.shape
    T = stride if n_groups is None else n_groups
    idx = np.full((rows, k), -1, np.int32)
    k_eff = lib().tomref_topk(_p(scores), stride, rows, T, k, order, _p(idx))
    if k_eff < 0:
        raise ValueError("tomref_topk: bad argument")
    return idx, k_eff


def dequant_gather(st: Store, idx: np.ndarray, k_eff: int, layer0: int = 0, fill=None):
    """idx: [n_layers][k] int32.  Returns (K_act, V_act) [n_layers][H_k][k*G][d] in
    cfg.out_dtype (uint16 bits for bf16/f16).  `fill`: value the buffers hold beforehand."""
    cfg = st.cfg
    idx = np.ascontiguousarray(idx, np.int32)
    nl, k = idx.shape
    shape = (nl, cfg.n_kv_heads, k * cfg.group_tokens, cfg.head_dim)
    dt = _np_dtype(cfg.out_dtype)
    ko = np.zeros(shape, dt) if fill is None else np.full(shape, fill, dt)
    vo = ko.copy()
    rc = lib().tomref_dequant_gather(C.byref(cfg), _p(st.codes), _p(st.scale), _p(st.zero),
                                     st.n_groups, layer0, nl, _p(idx), k, k_eff, _p(ko), _p(vo))
    if rc != 0:
        raise ValueError(f"tomref_dequant_gather failed rc={rc}")
    return ko, vo


def assemble_active(st: Store, idx: np.ndarray, k_eff: int, prefix_rows: int, sys_k=None, sys_v=None,
                    layer0: int = 0, fill=None):
    """Active KV with a system-token prefix: returns (K_act, V_act)
    [n_layers][H_k][prefix_rows + k*G][d] in cfg.out_dtype."""
    cfg = st.cfg
    idx = np.ascontiguousarray(idx, np.int32)
    nl, k = idx.shape
    shape = (nl, cfg.n_kv_heads, prefix_rows + k * cfg.group_tokens, cfg.head_dim)
    dt = _np_dtype(cfg.out_dtype)
    ko = np.zeros(shape, dt) if fill is None else np.full(shape, fill, dt)
    vo = ko.copy()
    rc = lib().tomref_assemble_active(C.byref(cfg), _p(st.codes), _p(st.scale), _p(st.zero),
                                      st.n_groups, layer0, nl, _p(idx), k, k_eff, prefix_rows,
                                      _p(sys_k), _p(sys_v), _p(ko), _p(vo))
    if rc != 0:
        raise ValueError(f"tomref_assemble_active failed rc={rc}")
    return ko, vo


def tile_view(st: Store, l: int, kv: int, t: int, h: int):
    """(packed codes [G][d*bits/8], scale, zero) views of one stored head tile."""
    cfg = st.cfg
    G, d = cfg.group_tokens, cfg.head_dim
    cb = lib().tomref_code_bytes_per_tile(G, d, cfg.bits)
    mt = lib().tomref_meta_per_tile(G, d, cfg.qgroup, cfg.qaxis)
    ti = ((l * 2 + kv) * cfg.capacity_groups + t) * cfg.n_kv_heads + h
    return (st.codes[ti * cb:(ti + 1) * cb].reshape(G, -1),
            st.scale[ti * mt:(ti + 1) * mt], st.zero[ti * mt:(ti + 1) * mt])
