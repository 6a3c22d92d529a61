"""Thin ctypes binding of libtom_oqm.so (the C ABI in include/tom_oqm.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory (`torch.empty`, `.data_ptr()`) and
for the current HIP stream, nothing else.  If the library has not been built,
importing this module raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtom_oqm.so")

# enums of include/tom_oqm.h
TOM_OK, TOM_ERR_INVALID_ARG, TOM_ERR_CAPACITY, TOM_ERR_UNSUPPORTED, TOM_ERR_NOT_BOUND, TOM_ERR_HIP = range(6)
TOM_F32, TOM_BF16, TOM_F16 = 0, 1, 2
TOM_QAXIS_HEAD_DIM, TOM_QAXIS_TOKENS = 0, 1
TOM_SIM_DOT, TOM_SIM_COSINE = 0, 1
TOM_ORDER_INDEX_ASC, TOM_ORDER_SCORE_DESC = 0, 1
TOM_SCORE_AUTO, TOM_SCORE_MEAN_QUERY, TOM_SCORE_TOKEN_GEMM = 0, 1, 2

_STATUS_NAMES = ["TOM_OK", "TOM_ERR_INVALID_ARG", "TOM_ERR_CAPACITY", "TOM_ERR_UNSUPPORTED",
                 "TOM_ERR_NOT_BOUND", "TOM_ERR_HIP"]

EXPORTS = ["tom_oqm_query_sizes", "tom_oqm_create", "tom_oqm_bind", "tom_oqm_reset",
           "tom_oqm_num_groups", "tom_oqm_set_num_groups", "tom_oqm_destroy", "tom_last_error",
           "tom_oqm_k_from_budget", "tom_oqm_quantize_append", "tom_oqm_score_workspace_bytes",
           "tom_oqm_score_groups", "tom_oqm_topk", "tom_oqm_dequant_gather",
           "tom_oqm_assemble_active", "tom_oqm_retrieve", "tom_oqm_retrieve_noalloc",
           "tom_oqm_static_scratch_bytes"]


class TomError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES[status] if 0 <= status < 6 else status}: {message}")
        self.status = status


class tom_oqm_config_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_kv_heads", "n_q_heads", "head_dim", "group_tokens", "qgroup", "qaxis",
        "bits", "capacity_groups", "in_dtype", "out_dtype", "sim", "meta_dtype")]


class tom_oqm_sizes_t(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("codes", "meta", "keys")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2510_18269_amd.build); "
            "there is no fallback implementation")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    cfgp = C.POINTER(tom_oqm_config_t)
    L.tom_oqm_query_sizes.argtypes = [cfgp, C.POINTER(tom_oqm_sizes_t)]
    L.tom_oqm_create.argtypes = [cfgp, C.POINTER(vp)]
    L.tom_oqm_bind.argtypes = [vp, vp, vp, vp]
    L.tom_oqm_reset.argtypes = [vp]
    L.tom_oqm_num_groups.argtypes = [vp]
    L.tom_oqm_set_num_groups.argtypes = [vp, i32]
    L.tom_oqm_destroy.argtypes = [vp]
    L.tom_oqm_destroy.restype = None
    L.tom_last_error.argtypes = []
    L.tom_last_error.restype = C.c_char_p
    L.tom_oqm_k_from_budget.argtypes = [i64, i32, i32]
    L.tom_oqm_quantize_append.argtypes = [vp, i32, i32, i32, vp, vp, vp, C.POINTER(i64), i32, vp,
                                          C.POINTER(i32)]
    L.tom_oqm_score_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    L.tom_oqm_score_workspace_bytes.restype = C.c_size_t
    L.tom_oqm_score_groups.argtypes = [vp, i32, i32, vp, i32, i32, vp, i64, vp, i32, vp,
                                       C.c_size_t, vp]
    L.tom_oqm_topk.argtypes = [vp, i64, i32, i32, i32, i32, vp, C.POINTER(i32), vp]
    L.tom_oqm_dequant_gather.argtypes = [vp, i32, i32, vp, i32, i32, vp, vp, vp]
    L.tom_oqm_assemble_active.argtypes = [vp, i32, i32, vp, i32, i32, i32, vp, vp, vp, vp, vp]
    L.tom_oqm_retrieve.argtypes = [vp, i32, i32, vp, i32, i32, i32, i32, vp, i64, vp, i32, vp, vp,
                                   vp, vp, vp, C.c_size_t, C.POINTER(i32), vp]
    L.tom_oqm_retrieve_noalloc.argtypes = [vp, i32, i32, vp, i32, i32, i32, i32, vp, i64, vp, i32, vp,
                                           vp, vp, vp, C.POINTER(i32), vp]
    L.tom_oqm_static_scratch_bytes.argtypes = []
    L.tom_oqm_static_scratch_bytes.restype = C.c_size_t
    for name in EXPORTS:
        fn = getattr(L, name)
        if name not in ("tom_oqm_destroy", "tom_last_error", "tom_oqm_score_workspace_bytes",
                        "tom_oqm_static_scratch_bytes"):
            fn.restype = i32
    return L


lib = _load()

_DTYPE_OF_TORCH = {torch.float32: TOM_F32, torch.bfloat16: TOM_BF16, torch.float16: TOM_F16}
_TORCH_OF_DTYPE = {v: k for k, v in _DTYPE_OF_TORCH.items()}


def tom_last_error() -> str:
    return lib.tom_last_error().decode()


def _check(status: int) -> None:
    if status != TOM_OK:
        raise TomError(status, tom_last_error())


def _ptr(t) -> int | None:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda, "device tensor expected"
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        # without a GPU only argument validation can run; it never reaches a launch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def tom_oqm_query_sizes(cfg: tom_oqm_config_t) -> tom_oqm_sizes_t:
    sizes = tom_oqm_sizes_t()
    _check(lib.tom_oqm_query_sizes(C.byref(cfg), C.byref(sizes)))
    return sizes


def tom_oqm_create(cfg: tom_oqm_config_t) -> int:
    h = C.c_void_p()
    _check(lib.tom_oqm_create(C.byref(cfg), C.byref(h)))
    return h.value


def tom_oqm_bind(h: int, codes, meta, keys) -> None:
    _check(lib.tom_oqm_bind(h, _ptr(codes), _ptr(meta), _ptr(keys)))


def tom_oqm_reset(h: int) -> None:
    _check(lib.tom_oqm_reset(h))


def tom_oqm_num_groups(h: int) -> int:
    return lib.tom_oqm_num_groups(h)


def tom_oqm_set_num_groups(h: int, n: int) -> None:
    _check(lib.tom_oqm_set_num_groups(h, n))


def tom_oqm_destroy(h: int) -> None:
    lib.tom_oqm_destroy(h)


def tom_oqm_k_from_budget(budget_tokens: int, group_tokens: int, stored_groups: int) -> int:
    return lib.tom_oqm_k_from_budget(budget_tokens, group_tokens, stored_groups)


def tom_oqm_quantize_append(h: int, layer0: int, n_layers: int, n_frames: int, k, v,
                            k_for_summary=None, strides=None, commit: bool = True,
                            stream=None) -> int:
    """k, v: device tensors (or raw device pointers).  `strides` = (frame, layer, head, token)
    in elements; None means a contiguous [n_frames][n_layers][H_k][G][d] tensor.
    Returns the first group slot written."""
    if strides is None:
        s = k.stride()
        assert k.dim() == 5 and s[4] == 1, "contiguous channel axis expected"
        strides = (s[0], s[1], s[2], s[3])
        assert tuple(v.stride()) == tuple(k.stride())
    sarr = (C.c_int64 * 4)(*strides)
    first = C.c_int32(-1)
    _check(lib.tom_oqm_quantize_append(h, layer0, n_layers, n_frames, _ptr(k), _ptr(v),
                                       _ptr(k_for_summary), sarr, 1 if commit else 0,
                                       _stream(stream), C.byref(first)))
    return first.value


def tom_oqm_score_workspace_bytes(h: int, n_layers: int, t_q: int, path: int = TOM_SCORE_AUTO,
                                  want_token_scores: bool = False) -> int:
    return lib.tom_oqm_score_workspace_bytes(h, n_layers, t_q, path, 1 if want_token_scores else 0)


def tom_oqm_score_groups(h: int, layer0: int, n_layers: int, q, t_q: int, scores,
                         score_stride: int, token_scores=None, path: int = TOM_SCORE_AUTO,
                         workspace=None, stream=None, q_dtype: int | None = None) -> None:
    if q_dtype is None:
        q_dtype = _DTYPE_OF_TORCH[q.dtype]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.tom_oqm_score_groups(h, layer0, n_layers, _ptr(q), q_dtype, t_q, _ptr(scores),
                                    score_stride, _ptr(token_scores), path, _ptr(workspace),
                                    ws_bytes, _stream(stream)))


def tom_oqm_topk(scores, score_stride: int, n_rows: int, n_groups: int, k: int, idx,
                 order: int = TOM_ORDER_INDEX_ASC, stream=None) -> int:
    """Returns k_eff = min(k, n_groups)."""
    k_eff = C.c_int32(-1)
    _check(lib.tom_oqm_topk(_ptr(scores), score_stride, n_rows, n_groups, k, order, _ptr(idx),
                            C.byref(k_eff), _stream(stream)))
    return k_eff.value


def tom_oqm_dequant_gather(h: int, layer0: int, n_layers: int, idx, k: int, k_eff: int, k_out,
                           v_out, stream=None) -> None:
    _check(lib.tom_oqm_dequant_gather(h, layer0, n_layers, _ptr(idx), k, k_eff, _ptr(k_out),
                                      _ptr(v_out), _stream(stream)))


def tom_oqm_assemble_active(h: int, layer0: int, n_layers: int, idx, k: int, k_eff: int,
                            prefix_rows: int, sys_k, sys_v, k_out, v_out, stream=None) -> None:
    _check(lib.tom_oqm_assemble_active(h, layer0, n_layers, _ptr(idx), k, k_eff, prefix_rows,
                                       _ptr(sys_k), _ptr(sys_v), _ptr(k_out), _ptr(v_out),
                                       _stream(stream)))


def tom_oqm_retrieve(h: int, layer0: int, n_layers: int, q, t_q: int, k: int, scores,
                     score_stride: int, idx, k_out, v_out, workspace, path: int = TOM_SCORE_AUTO,
                     prefix_rows: int = 0, sys_k=None, sys_v=None, stream=None,
                     q_dtype: int | None = None) -> int:
    """score -> top-k -> assemble in one call.  Returns k_eff."""
    if q_dtype is None:
        q_dtype = _DTYPE_OF_TORCH[q.dtype]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    k_eff = C.c_int32(-1)
    _check(lib.tom_oqm_retrieve(h, layer0, n_layers, _ptr(q), q_dtype, t_q, k, path, _ptr(scores),
                                score_stride, _ptr(idx), prefix_rows, _ptr(sys_k), _ptr(sys_v),
                                _ptr(k_out), _ptr(v_out), _ptr(workspace), ws_bytes,
                                C.byref(k_eff), _stream(stream)))
    return k_eff.value


def tom_oqm_retrieve_noalloc(h: int, layer0: int, n_layers: int, q, t_q: int, k: int, scores,
                             score_stride: int, idx, k_out, v_out, path: int = TOM_SCORE_AUTO,
                             prefix_rows: int = 0, sys_k=None, sys_v=None, stream=None,
                             q_dtype: int | None = None) -> int:
    """tom_oqm_retrieve without a workspace: the score scratch is the library's static array."""
    if q_dtype is None:
        q_dtype = _DTYPE_OF_TORCH[q.dtype]
    k_eff = C.c_int32(-1)
    _check(lib.tom_oqm_retrieve_noalloc(h, layer0, n_layers, _ptr(q), q_dtype, t_q, k, path,
                                        _ptr(scores), score_stride, _ptr(idx), prefix_rows,
                                        _ptr(sys_k), _ptr(sys_v), _ptr(k_out), _ptr(v_out),
                                        C.byref(k_eff), _stream(stream)))
    return k_eff.value


def tom_oqm_static_scratch_bytes() -> int:
    return lib.tom_oqm_static_scratch_bytes()


# --------------------------------------------------------------------------- convenience
def make_config(n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup, capacity_groups,
                qaxis=TOM_QAXIS_HEAD_DIM, bits=4, in_dtype=TOM_BF16, out_dtype=TOM_BF16,
                sim=TOM_SIM_COSINE, meta_dtype=TOM_F32) -> tom_oqm_config_t:
    return tom_oqm_config_t(n_layers, n_kv_heads, n_q_heads, head_dim, group_tokens, qgroup,
                            qaxis, bits, capacity_groups, in_dtype, out_dtype, sim, meta_dtype)


@dataclass
class Memory:
    """A handle plus the torch tensors that back its storage (allocation only: all work
    goes through the tom_oqm_* calls above)."""
    cfg: tom_oqm_config_t
    handle: int
    codes: torch.Tensor
    meta: torch.Tensor     # (scale, zero) pairs, float32 or bfloat16 (cfg.meta_dtype)
    keys: torch.Tensor

    @staticmethod
    def allocate(cfg: tom_oqm_config_t, device="cuda:0") -> "Memory":
        sizes = tom_oqm_query_sizes(cfg)
        h = tom_oqm_create(cfg)
        codes = torch.empty(sizes.codes, dtype=torch.uint8, device=device)
        if cfg.meta_dtype == TOM_BF16:
            meta = torch.empty(sizes.meta // 2, dtype=torch.bfloat16, device=device)
        else:
            meta = torch.empty(sizes.meta // 4, dtype=torch.float32, device=device)
        keys = torch.empty(sizes.keys // 4, dtype=torch.float32, device=device)
        tom_oqm_bind(h, codes, meta, keys)
        return Memory(cfg, h, codes, meta, keys)

    @property
    def n_groups(self) -> int:
        return tom_oqm_num_groups(self.handle)

    def out_torch_dtype(self) -> torch.dtype:
        return _TORCH_OF_DTYPE[self.cfg.out_dtype]

    def close(self) -> None:
        if self.handle:
            tom_oqm_destroy(self.handle)
            self.handle = 0
