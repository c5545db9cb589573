"""ctypes binding of libcritiprefill.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors used purely as device buffers; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: a missing library or a non-zero status raises.
"""
from __future__ import annotations

import ctypes
import math
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcritiprefill.so")
_lib = None

CP_DTYPE_FP32, CP_DTYPE_BF16 = 0, 1
EXPORTS = ["critiprefill_list_len", "critiprefill_workspace_bytes", "critiprefill_estimate",
           "critiprefill_estimate_static", "critiprefill_select", "critiprefill_sparse_attn", "critiprefill_select_shared",
           "critiprefill_sparse_attn_shared", "critiprefill_dense_causal_attn",
           "critiprefill_strerror", "critiprefill_version"]


class Params(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("segment_size", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("budget_blocks", ctypes.c_int32), ("local_blocks", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("attn_scale", ctypes.c_float), ("score_scale", ctypes.c_float),
                ("alpha", ctypes.c_float), ("softmax_domain", ctypes.c_int32),
                ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3)]


class CritiPrefillError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({strerror(status)})")


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} not built: run `python -m paper_2409_12490_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    P = ctypes.POINTER(Params)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.critiprefill_list_len.argtypes = [P]; lib.critiprefill_list_len.restype = ctypes.c_int32
    lib.critiprefill_workspace_bytes.argtypes = [P]; lib.critiprefill_workspace_bytes.restype = sz
    lib.critiprefill_estimate.argtypes = [P, vp, vp, vp, vp, vp, sz, vp]; lib.critiprefill_estimate.restype = ctypes.c_int
    lib.critiprefill_estimate_static.argtypes = [P, vp, vp, vp, vp, vp]; lib.critiprefill_estimate_static.restype = ctypes.c_int
    lib.critiprefill_select.argtypes = [P, vp, vp, vp, vp]; lib.critiprefill_select.restype = ctypes.c_int
    lib.critiprefill_sparse_attn.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp]; lib.critiprefill_sparse_attn.restype = ctypes.c_int
    lib.critiprefill_select_shared.argtypes = [P, vp, vp, vp, vp]; lib.critiprefill_select_shared.restype = ctypes.c_int
    lib.critiprefill_sparse_attn_shared.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp]; lib.critiprefill_sparse_attn_shared.restype = ctypes.c_int
    lib.critiprefill_dense_causal_attn.argtypes = [P, vp, vp, vp, vp, vp, vp]; lib.critiprefill_dense_causal_attn.restype = ctypes.c_int
    lib.critiprefill_strerror.argtypes = [ctypes.c_int]; lib.critiprefill_strerror.restype = ctypes.c_char_p
    lib.critiprefill_version.argtypes = []; lib.critiprefill_version.restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().critiprefill_strerror(status).decode()


def version() -> int:
    return load().critiprefill_version()


def make_params(q: torch.Tensor, k: torch.Tensor, segment_size: int, block_size: int, budget_blocks: int,
                local_blocks: int = 0, out: torch.Tensor | None = None, attn_scale: float = 0.0,
                score_scale: float = 0.0, alpha: float = 1.0, softmax_domain: int = 0) -> Params:
    """Fill the parameter block from tensor shapes/strides (q [B,Hq,n,d], k [B,Hkv,n,d])."""
    p = Params()
    p.batch, p.n_q_heads, p.seq_len, p.head_dim = q.shape[0], q.shape[1], q.shape[2], q.shape[3]
    p.n_kv_heads = k.shape[1]
    p.segment_size, p.block_size = segment_size, block_size
    p.budget_blocks, p.local_blocks = budget_blocks, local_blocks
    if q.dtype == torch.bfloat16:
        p.dtype = CP_DTYPE_BF16
    elif q.dtype == torch.float32:
        p.dtype = CP_DTYPE_FP32
    else:
        raise TypeError(f"unsupported dtype {q.dtype}")
    p.attn_scale, p.score_scale, p.alpha, p.softmax_domain = attn_scale, score_scale, alpha, softmax_domain
    if q.stride(3) != 1 or k.stride(3) != 1:
        raise ValueError("channel stride must be 1")
    for i in range(3):
        p.q_stride[i] = q.stride(i)
        p.kv_stride[i] = k.stride(i)
        p.o_stride[i] = (out if out is not None else q).stride(i)
    return p


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise CritiPrefillError(status, where)


def critiprefill_list_len(p: Params) -> int:
    return load().critiprefill_list_len(ctypes.byref(p))


def critiprefill_workspace_bytes(p: Params) -> int:
    return load().critiprefill_workspace_bytes(ctypes.byref(p))


def critiprefill_estimate(p, q, k, prev_scores, scores, workspace, stream=None):
    _check(load().critiprefill_estimate(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(prev_scores), _ptr(scores),
                                        _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _stream(stream)), "critiprefill_estimate")


def critiprefill_estimate_static(p, q, k, prev_scores, scores, stream=None):
    _check(load().critiprefill_estimate_static(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(prev_scores), _ptr(scores),
                                               _stream(stream)), "critiprefill_estimate_static")


def critiprefill_select(p, scores, block_idx, block_cnt, stream=None):
    _check(load().critiprefill_select(ctypes.byref(p), _ptr(scores), _ptr(block_idx), _ptr(block_cnt),
                                      _stream(stream)), "critiprefill_select")


def critiprefill_sparse_attn(p, q, k, v, block_idx, block_cnt, out, lse=None, stream=None):
    _check(load().critiprefill_sparse_attn(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(block_idx),
                                           _ptr(block_cnt), _ptr(out), _ptr(lse), _stream(stream)),
           "critiprefill_sparse_attn")


def critiprefill_select_shared(p, scores, block_idx, block_cnt, stream=None):
    _check(load().critiprefill_select_shared(ctypes.byref(p), _ptr(scores), _ptr(block_idx), _ptr(block_cnt),
                                             _stream(stream)), "critiprefill_select_shared")


def critiprefill_sparse_attn_shared(p, q, k, v, block_idx, block_cnt, out, lse=None, stream=None):
    _check(load().critiprefill_sparse_attn_shared(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(block_idx),
                                                  _ptr(block_cnt), _ptr(out), _ptr(lse), _stream(stream)),
           "critiprefill_sparse_attn_shared")


def critiprefill_dense_causal_attn(p, q, k, v, out, lse=None, stream=None):
    _check(load().critiprefill_dense_causal_attn(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse),
                                                 _stream(stream)), "critiprefill_dense_causal_attn")


# ---- buffer helpers (device memory only; no arithmetic) -----------------------------------------
def n_segments(p: Params) -> int:
    return -(-p.seq_len // p.segment_size)


def n_blocks(p: Params) -> int:
    return -(-p.seq_len // p.block_size)


def alloc_scores(p: Params, device="cuda") -> torch.Tensor:
    return torch.empty((p.batch, p.n_q_heads, n_segments(p), n_blocks(p)), dtype=torch.float32, device=device)


def alloc_lists(p: Params, device="cuda"):
    ll = critiprefill_list_len(p)
    idx = torch.empty((p.batch, p.n_q_heads, n_segments(p), ll), dtype=torch.int32, device=device)
    cnt = torch.empty((p.batch, p.n_q_heads, n_segments(p)), dtype=torch.int32, device=device)
    return idx, cnt


def alloc_shared_lists(p: Params, device="cuda"):
    """Lists of critiprefill_select_shared: one per (batch, KV head, segment)."""
    ll = critiprefill_list_len(p)
    idx = torch.empty((p.batch, p.n_kv_heads, n_segments(p), ll), dtype=torch.int32, device=device)
    cnt = torch.empty((p.batch, p.n_kv_heads, n_segments(p)), dtype=torch.int32, device=device)
    return idx, cnt


def alloc_workspace(p: Params, device="cuda") -> torch.Tensor:
    return torch.empty((max(16, critiprefill_workspace_bytes(p)),), dtype=torch.uint8, device=device)
