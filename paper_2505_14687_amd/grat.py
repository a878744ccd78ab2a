"""Thin ctypes binding over libgrat.so: argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the attention path
runs inside the library's kernels.  There is no fallback: if libgrat.so has not been built
(python -m paper_2505_14687_amd.build) every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

from .build import LIB_PATH

GRAT_OK = 0
PATTERNS = {"block": 0, "cross": 1, "cross_planes": 2, "dense": 3}
DTYPES = {torch.bfloat16: 0, torch.float32: 1, torch.float16: 2}
EXPORTS = ("grat_block_list_shape", "grat_build_block_lists", "grat_validate_block_lists", "grat_attention_fwd",
           "grat_attention_global_fwd", "grat_attention_packed_fwd", "grat_dense_attention_fwd",
           "grat_status_string", "grat_probe_mfma")

_i32, _i64, _f32, _vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
_pi32 = ctypes.POINTER(ctypes.c_int32)
_lib = None


class GratError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().grat_status_string(status).decode()
        super().__init__(f"{where}: status {status} ({msg})")


def lib() -> ctypes.CDLL:
    """Load libgrat.so (once).  Raises if it is not there: there is no other implementation."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2505_14687_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        L.grat_block_list_shape.argtypes = [_i32, _pi32, _pi32, _i32, _pi32, _pi32, _pi32]
        L.grat_block_list_shape.restype = _i32
        L.grat_build_block_lists.argtypes = [_i32, _pi32, _pi32, _i32, _pi32, _vp, _vp, _i32, _vp]
        L.grat_build_block_lists.restype = _i32
        L.grat_validate_block_lists.argtypes = [_i32, _pi32, _pi32, _vp, _vp, _i32, _vp, _vp]
        L.grat_validate_block_lists.restype = _i32
        L.grat_attention_fwd.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i64, _i64, _i64,
                                         _f32, _i32, _pi32, _pi32, _vp, _vp, _i32, _vp]
        L.grat_attention_fwd.restype = _i32
        L.grat_attention_global_fwd.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i64, _i64,
                                                _i64, _f32, _i32, _i32, _i32, _pi32, _pi32, _vp, _vp,
                                                _i32, _vp]
        L.grat_attention_global_fwd.restype = _i32
        L.grat_attention_packed_fwd.argtypes = [_vp, _vp, _i32, _i32, _i32, _i32, _f32, _i32, _i32, _i32,
                                                _pi32, _pi32, _vp, _vp, _i32, _vp]
        L.grat_attention_packed_fwd.restype = _i32
        L.grat_dense_attention_fwd.argtypes = [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i64, _i32,
                                               _i64, _i64, _i64, _f32, _vp]
        L.grat_dense_attention_fwd.restype = _i32
        L.grat_status_string.argtypes = [_i32]
        L.grat_status_string.restype = ctypes.c_char_p
        L.grat_probe_mfma.argtypes = [_i32, _i32, _vp, _i32, _i32, _vp]
        L.grat_probe_mfma.restype = _i32
        _lib = L
    return _lib


def _ivec(values: Optional[Sequence[int]]):
    if values is None:
        return None
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def _pattern_id(pattern) -> int:
    return PATTERNS[pattern] if isinstance(pattern, str) else int(pattern)


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def grat_block_list_shape(grid: Sequence[int], group: Sequence[int], pattern,
                          radius: Optional[Sequence[int]] = None) -> Tuple[int, int]:
    """(num_groups, max_kv) for a pattern; host only."""
    g, mk = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib().grat_block_list_shape(len(grid), _ivec(grid), _ivec(group), _pattern_id(pattern),
                                     _ivec(radius), ctypes.byref(g), ctypes.byref(mk))
    if st != GRAT_OK:
        raise GratError(st, "grat_block_list_shape")
    return g.value, mk.value


def grat_build_block_lists(grid: Sequence[int], group: Sequence[int], pattern,
                           radius: Optional[Sequence[int]] = None, device="cuda",
                           max_kv: Optional[int] = None, stream=None):
    """Build the lists on the GPU.  Returns (kv_count int32 [G], kv_index int32 [G, max_kv])."""
    G, need = grat_block_list_shape(grid, group, pattern, radius)
    max_kv = need if max_kv is None else int(max_kv)
    kv_count = torch.empty(G, dtype=torch.int32, device=device)
    kv_index = torch.empty((G, max(max_kv, 1)), dtype=torch.int32, device=device)
    st = lib().grat_build_block_lists(len(grid), _ivec(grid), _ivec(group), _pattern_id(pattern),
                                      _ivec(radius), kv_count.data_ptr(), kv_index.data_ptr(),
                                      max_kv, _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_build_block_lists")
    return kv_count, kv_index


LIST_BAD_COUNT, LIST_BAD_ENTRY, LIST_BAD_PADDING = 1, 2, 4


def grat_validate_block_lists(grid: Sequence[int], group: Sequence[int], kv_count, kv_index, stream=None):
    """Checks lists on the GPU; returns a device int32 tensor [1]: 0, or the OR of the LIST_BAD_* flags
    (read it after synchronising with the stream, e.g. with .item())."""
    _check_lists(kv_count, kv_index, _num_groups(grid, group), kv_count.device)
    if not kv_count.is_cuda:
        raise ValueError("libgrat works on device memory only")
    status = torch.empty(1, dtype=torch.int32, device=kv_count.device)
    st = lib().grat_validate_block_lists(len(grid), _ivec(grid), _ivec(group), kv_count.data_ptr(),
                                         kv_index.data_ptr(), int(kv_index.shape[1]), status.data_ptr(),
                                         _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_validate_block_lists")
    return status


def _check_qkvo(Q, K, V, O):
    if Q.dim() != 4:
        raise ValueError("expected [B, H, N, d] tensors (any strides with d contiguous)")
    for name, t in (("K", K), ("V", V), ("O", O)):
        if t.shape != Q.shape or t.dtype != Q.dtype or t.stride() != Q.stride() or t.device != Q.device:
            raise ValueError(f"{name} must match Q in shape, dtype, strides and device")
    if Q.stride(3) != 1:
        raise ValueError("the head_dim axis must be contiguous")
    if Q.dtype not in DTYPES:
        raise ValueError(f"unsupported dtype {Q.dtype}")
    if not Q.is_cuda:
        raise ValueError("libgrat works on device memory only")


def _num_groups(grid: Sequence[int], group: Sequence[int]) -> int:
    if len(grid) != len(group) or not 1 <= len(grid) <= 3 or min(list(grid) + list(group)) < 1:
        raise ValueError("grid and group must have the same 1 to 3 positive extents")
    n = 1
    for t, g in zip(grid, group):
        n *= -(-int(t) // int(g))
    return n


def _check_sequence(seq_len: int, grid: Sequence[int], n_global: int = 0):
    """The kernels address prod(grid) + n_global token rows: the tensors must hold exactly that many."""
    n = 1
    for t in grid:
        n *= int(t)
    if int(n_global) < 0 or seq_len != n + int(n_global):
        raise ValueError(f"sequence length {seq_len} does not match prod(grid) + n_global = {n} + {n_global}")


def _check_lists(kv_count, kv_index, num_groups: int, device):
    """Block lists as the library reads them: int32, contiguous, [G] and [G, max_kv], on the tensors' device."""
    for name, t in (("kv_count", kv_count), ("kv_index", kv_index)):
        if not isinstance(t, torch.Tensor) or t.dtype != torch.int32:
            raise ValueError(f"{name} must be an int32 tensor")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if kv_count.dim() != 1 or kv_count.numel() != num_groups:
        raise ValueError(f"kv_count must have shape [{num_groups}] (one entry per group)")
    if kv_index.dim() != 2 or kv_index.shape[0] != num_groups or kv_index.shape[1] < 1:
        raise ValueError(f"kv_index must have shape [{num_groups}, max_kv]")
    for name, t in (("kv_count", kv_count), ("kv_index", kv_index)):
        if t.device != device:
            raise ValueError(f"{name} must live on the tensors' device ({device})")


def grat_attention_fwd(Q, K, V, scale: float, grid: Sequence[int], group: Sequence[int],
                       kv_count, kv_index, out=None, stream=None):
    """O = softmax(scale * Q K^T over the listed KV groups) V.  Q, K, V: [B, H, N, d] views."""
    O = torch.empty_like(Q) if out is None else out
    if Q.dim() == 4:
        _check_sequence(Q.shape[2], grid)
        _check_lists(kv_count, kv_index, _num_groups(grid, group), Q.device)
    _check_qkvo(Q, K, V, O)
    B, H, N, d = Q.shape
    st = lib().grat_attention_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                  DTYPES[Q.dtype], B, H, d, Q.stride(0), Q.stride(1), Q.stride(2),
                                  float(scale), len(grid), _ivec(grid), _ivec(group),
                                  kv_count.data_ptr(), kv_index.data_ptr(), int(kv_index.shape[1]),
                                  _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_attention_fwd")
    return O


def grat_attention_global_fwd(Q, K, V, scale: float, n_global: int, global_first: bool,
                              grid: Sequence[int], group: Sequence[int], kv_count, kv_index,
                              out=None, stream=None):
    """Joint sequence of n_global prompt tokens and the grid tokens; Q, K, V: [B, H, n_global + N, d]."""
    O = torch.empty_like(Q) if out is None else out
    if Q.dim() == 4:
        _check_sequence(Q.shape[2], grid, n_global)
        _check_lists(kv_count, kv_index, _num_groups(grid, group), Q.device)
    _check_qkvo(Q, K, V, O)
    B, H, L, d = Q.shape
    st = lib().grat_attention_global_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                         DTYPES[Q.dtype], B, H, d, Q.stride(0), Q.stride(1),
                                         Q.stride(2), float(scale), int(n_global), int(bool(global_first)),
                                         len(grid), _ivec(grid), _ivec(group), kv_count.data_ptr(),
                                         kv_index.data_ptr(), int(kv_index.shape[1]),
                                         _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_attention_global_fwd")
    return O


def grat_attention_packed_fwd(QKV, scale: float, grid: Sequence[int], group: Sequence[int], kv_count,
                              kv_index, n_global: int = 0, global_first: bool = True, out=None,
                              stream=None):
    """QKV: contiguous [B, L, 3, H, d] (L = n_global + grid tokens); returns O as [B, L, H, d]."""
    if QKV.dim() != 5 or QKV.shape[2] != 3 or not QKV.is_contiguous():
        raise ValueError("expected a contiguous [B, L, 3, H, d] tensor")
    B, L, _, H, d = QKV.shape
    _check_sequence(L, grid, n_global)
    _check_lists(kv_count, kv_index, _num_groups(grid, group), QKV.device)
    if QKV.dtype not in DTYPES or not QKV.is_cuda:
        raise ValueError("libgrat works on bf16 / fp16 / fp32 device memory only")
    O = torch.empty((B, L, H, d), dtype=QKV.dtype, device=QKV.device) if out is None else out
    if O.shape != (B, L, H, d) or O.dtype != QKV.dtype or not O.is_contiguous() or O.device != QKV.device:
        raise ValueError("out must be a contiguous [B, L, H, d] tensor of QKV's dtype and device")
    st = lib().grat_attention_packed_fwd(QKV.data_ptr(), O.data_ptr(), DTYPES[QKV.dtype], B, H, d,
                                         float(scale), int(n_global), int(bool(global_first)),
                                         len(grid), _ivec(grid), _ivec(group), kv_count.data_ptr(),
                                         kv_index.data_ptr(), int(kv_index.shape[1]),
                                         _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_attention_packed_fwd")
    return O


def grat_dense_attention_fwd(Q, K, V, scale: float, out=None, stream=None):
    """O = softmax(scale * Q K^T) V over the whole sequence."""
    O = torch.empty_like(Q) if out is None else out
    _check_qkvo(Q, K, V, O)
    B, H, N, d = Q.shape
    st = lib().grat_dense_attention_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                        DTYPES[Q.dtype], B, H, N, d, Q.stride(0), Q.stride(1),
                                        Q.stride(2), float(scale), _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_dense_attention_fwd")
    return O
