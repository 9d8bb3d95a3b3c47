"""Thin ctypes binding of the C ABI in include/dart.h.

Argument marshalling only: every step runs in the HIP kernels of
libdart_hip.so.  PyTorch supplies device memory and the current stream.  If the
library is missing this module raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch


LIB = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdart_hip.so")

DART_OK = 0
DART_ERR_NULL, DART_ERR_SHAPE, DART_ERR_BUDGET, DART_ERR_DTYPE = -1, -2, -3, -4
DART_ERR_WORKSPACE, DART_ERR_ALIGN, DART_ERR_HIP, DART_ERR_DEVICE = -5, -6, -7, -8
DART_ERR_STATIC_LIMIT = -9
DART_F32, DART_BF16 = 0, 1
DART_PIVOT_MAX_L1, DART_PIVOT_MIN_L1, DART_PIVOT_GIVEN, DART_PIVOT_RANDOM = 0, 1, 2, 3
DART_SCORE_PER_PIVOT, DART_SCORE_MIN, DART_SCORE_MAX = 0, 1, 2

EXPORTS = ("dart_workspace_bytes", "dart_select_pivots", "dart_duplication_scores",
           "dart_topk_keep", "dart_gather_compact", "dart_compact_sequences", "dart_reduce",
           "dart_reduce_profiled", "dart_reduce_static", "dart_static_scratch_bytes",
           "dart_device_status_static", "dart_probe_mfma_dot32", "dart_score_tile_shape",
           "dart_score_tile_shape_first_read", "dart_reduce_with_norms",
           "dart_device_status", "dart_score_tolerance", "dart_strerror")


class DartDesc(C.Structure):
    """Mirror of `struct dart_desc`."""
    _fields_ = [("B", C.c_int32), ("D", C.c_int32), ("P", C.c_int32), ("N", C.c_int32),
                ("cu_seqlens", C.c_void_p), ("total_N", C.c_int32), ("max_N", C.c_int32),
                ("ld", C.c_int64), ("dtype", C.c_int32), ("K", C.c_int32),
                ("keep_num", C.c_int32), ("keep_den", C.c_int32), ("pivot_mode", C.c_int32),
                ("score_mode", C.c_int32), ("P_ext", C.c_int32), ("ext_ld", C.c_int64),
                ("ext_pivots", C.c_void_p), ("span_start", C.c_void_p), ("X_rows", C.c_int32),
                ("seed", C.c_uint64)]


class DartRowTensor(C.Structure):
    """Mirror of `struct dart_row_tensor`."""
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("row_bytes", C.c_int64),
                ("src_ld_bytes", C.c_int64), ("dst_ld_bytes", C.c_int64)]


class DartError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise RuntimeError(f"{LIB} is missing: run `python -m paper_2502_11494_amd.build`")
        L = C.CDLL(LIB)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        dp = C.POINTER(DartDesc)
        L.dart_workspace_bytes.argtypes = [dp]
        L.dart_workspace_bytes.restype = sz
        L.dart_select_pivots.argtypes = [dp, vp, vp, i32, i64, vp, vp, vp, sz, vp]
        L.dart_duplication_scores.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.dart_topk_keep.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dart_gather_compact.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dart_compact_sequences.argtypes = [dp, vp, vp, i32, C.POINTER(DartRowTensor), vp, i32,
                                             i64, vp, i64, vp, vp, vp, sz, vp]
        L.dart_reduce.argtypes = [dp, vp, vp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dart_reduce_profiled.argtypes = L.dart_reduce.argtypes + [C.POINTER(vp)]
        L.dart_reduce_with_norms.argtypes = [dp, vp, vp, i32, i64, vp, C.c_double, vp, vp, vp, vp,
                                             vp, vp, vp, vp, sz, vp]
        L.dart_device_status.argtypes = [dp, vp, vp]
        L.dart_reduce_static.argtypes = [dp, vp, vp, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp]
        L.dart_score_tile_shape.argtypes = [dp, C.POINTER(i32), C.POINTER(i32)]
        L.dart_score_tile_shape_first_read.argtypes = [dp, C.POINTER(i32), C.POINTER(i32)]
        L.dart_static_scratch_bytes.argtypes = []
        L.dart_static_scratch_bytes.restype = sz
        L.dart_device_status_static.argtypes = [dp, vp]
        L.dart_probe_mfma_dot32.argtypes = [vp, vp, vp, i32, vp]
        for name in ("dart_select_pivots", "dart_duplication_scores", "dart_topk_keep",
                     "dart_gather_compact", "dart_compact_sequences", "dart_reduce",
                     "dart_reduce_profiled", "dart_device_status", "dart_reduce_static",
                     "dart_device_status_static", "dart_probe_mfma_dot32",
                     "dart_score_tile_shape", "dart_score_tile_shape_first_read",
                     "dart_reduce_with_norms"):
            getattr(L, name).restype = C.c_int
        L.dart_score_tolerance.argtypes = [i32]
        L.dart_score_tolerance.restype = C.c_double
        L.dart_strerror.argtypes = [C.c_int]
        L.dart_strerror.restype = C.c_char_p
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().dart_strerror(int(status)).decode()


def score_tolerance(dtype: int) -> float:
    return float(lib().dart_score_tolerance(int(dtype)))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def make_desc(B: int, D: int, P: int, dtype: int, *, N: int = 0, K: int = 0, keep_num: int = 0,
              keep_den: int = 1, cu_seqlens: Optional[torch.Tensor] = None, total_N: int = 0,
              max_N: int = 0, ld: Optional[int] = None,
              pivot_mode: int = DART_PIVOT_MAX_L1,
              score_mode: int = DART_SCORE_PER_PIVOT,
              ext_pivots: Optional[torch.Tensor] = None, P_ext: int = 0,
              ext_ld: Optional[int] = None, span_start: Optional[torch.Tensor] = None,
              X_rows: int = 0, seed: int = 0) -> DartDesc:
    d = DartDesc()
    d.B, d.D, d.P, d.N = B, D, P, N
    d.cu_seqlens = None if cu_seqlens is None else cu_seqlens.data_ptr()
    d.total_N, d.max_N = total_N, max_N
    d.ld = D if ld is None else ld
    d.dtype, d.K, d.keep_num, d.keep_den = dtype, K, keep_num, keep_den
    d.pivot_mode, d.score_mode = pivot_mode, score_mode
    d.P_ext = P_ext
    if ext_pivots is not None:  # a tensor, or a raw device address
        d.ext_pivots = ext_pivots.data_ptr() if hasattr(ext_pivots, "data_ptr") else int(ext_pivots)
    d.ext_ld = (D if ext_ld is None else ext_ld) if P_ext > 0 else 0
    if span_start is not None:  # a tensor, or a raw device address
        d.span_start = (span_start.data_ptr() if hasattr(span_start, "data_ptr")
                        else int(span_start))
    d.X_rows = X_rows
    d.seed = seed & (2**64 - 1)
    # the descriptor holds raw device addresses: keep their tensors alive with it
    d._keepalive = (cu_seqlens, ext_pivots, span_start)
    return d


def dart_workspace_bytes(desc: DartDesc) -> int:
    return int(lib().dart_workspace_bytes(C.byref(desc)))


def alloc_workspace(desc: DartDesc, device="cuda") -> torch.Tensor:
    n = dart_workspace_bytes(desc)
    if n == 0:
        raise DartError(DART_ERR_SHAPE, "dart_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _check(status: int, where: str):
    if status != DART_OK:
        raise DartError(status, where)


def dart_select_pivots(desc, X, piv, ws, *, crit=None, crit_D=0, crit_ld=0, l1_out=None,
                       stream=None):
    _check(lib().dart_select_pivots(C.byref(desc), _ptr(X), _ptr(crit), crit_D, crit_ld,
                                    _ptr(piv), _ptr(l1_out), _ptr(ws), ws.numel(),
                                    _stream(stream)), "dart_select_pivots")


def dart_duplication_scores(desc, X, piv, S, ws, *, stream=None):
    _check(lib().dart_duplication_scores(C.byref(desc), _ptr(X), _ptr(piv), _ptr(S), _ptr(ws),
                                         ws.numel(), _stream(stream)), "dart_duplication_scores")


def dart_topk_keep(desc, S, piv, keep, ws, *, X=None, cu_keep=None, stream=None):
    _check(lib().dart_topk_keep(C.byref(desc), _ptr(S), _ptr(piv), _ptr(X), _ptr(keep),
                                _ptr(cu_keep), _ptr(ws), ws.numel(), _stream(stream)),
           "dart_topk_keep")


def dart_gather_compact(desc, X, keep, Y, ws, *, pos=None, pos_out=None, stream=None):
    _check(lib().dart_gather_compact(C.byref(desc), _ptr(X), _ptr(pos), _ptr(keep), _ptr(Y),
                                     _ptr(pos_out), _ptr(ws), ws.numel(), _stream(stream)),
           "dart_gather_compact")


def dart_compact_sequences(desc, seq_cu, keep, tensors, seq_cu_out, row_map, ws, *, pos=None,
                           pos_out=None, stream=None):
    """tensors: list of (src, dst) 2-D tensors with contiguous rows (any row stride).
    pos / pos_out: [planes, rows] int64 tensors (plane-major), or None."""
    arr = (DartRowTensor * max(len(tensors), 1))()
    for i, (src, dst) in enumerate(tensors):
        esz = src.element_size()
        arr[i] = DartRowTensor(src.data_ptr(), dst.data_ptr(), src.shape[1] * esz,
                               src.stride(0) * esz, dst.stride(0) * esz)
    planes = 0 if pos is None else pos.shape[0]
    _check(lib().dart_compact_sequences(
        C.byref(desc), _ptr(seq_cu), _ptr(keep), len(tensors), arr, _ptr(pos), planes,
        0 if pos is None else pos.stride(0), _ptr(pos_out),
        0 if pos_out is None else pos_out.stride(0), _ptr(seq_cu_out), _ptr(row_map), _ptr(ws),
        ws.numel(), _stream(stream)), "dart_compact_sequences")


def dart_reduce(desc, X, Y, keep, ws, *, crit=None, crit_D=0, crit_ld=0, pos=None, pos_out=None,
                cu_keep=None, piv_out=None, S_out=None, stream=None):
    _check(lib().dart_reduce(C.byref(desc), _ptr(X), _ptr(crit), crit_D, crit_ld, _ptr(pos),
                             _ptr(Y), _ptr(pos_out), _ptr(keep), _ptr(cu_keep), _ptr(piv_out),
                             _ptr(S_out), _ptr(ws), ws.numel(), _stream(stream)), "dart_reduce")


def dart_reduce_with_norms(desc, X, Y, keep, ws, l1, l1_rel_err, *, crit=None, crit_D=0,
                           crit_ld=0, pos=None, pos_out=None, cu_keep=None, piv_out=None,
                           S_out=None, stream=None):
    """dart_reduce without its norm pass: l1 holds the criterion norms, good to l1_rel_err."""
    _check(lib().dart_reduce_with_norms(C.byref(desc), _ptr(X), _ptr(crit), crit_D, crit_ld,
                                        _ptr(l1), float(l1_rel_err), _ptr(pos), _ptr(Y),
                                        _ptr(pos_out), _ptr(keep), _ptr(cu_keep), _ptr(piv_out),
                                        _ptr(S_out), _ptr(ws), ws.numel(), _stream(stream)),
           "dart_reduce_with_norms")


def dart_reduce_static(desc, X, Y, keep, *, crit=None, crit_D=0, crit_ld=0, pos=None,
                       pos_out=None, cu_keep=None, piv_out=None, S_out=None, stream=None):
    """dart_reduce on the library's built-in scratch buffer: no workspace, no allocation."""
    _check(lib().dart_reduce_static(C.byref(desc), _ptr(X), _ptr(crit), crit_D, crit_ld,
                                    _ptr(pos), _ptr(Y), _ptr(pos_out), _ptr(keep),
                                    _ptr(cu_keep), _ptr(piv_out), _ptr(S_out), _stream(stream)),
           "dart_reduce_static")


def dart_score_tile_shape(desc) -> tuple:
    """(waves per workgroup, groups of them) of the score kernel for this descriptor; (0, 0)
    for fp32."""
    w, ks = C.c_int32(0), C.c_int32(0)
    _check(lib().dart_score_tile_shape(C.byref(desc), C.byref(w), C.byref(ks)),
           "dart_score_tile_shape")
    return int(w.value), int(ks.value)


def dart_score_tile_shape_first_read(desc) -> tuple:
    """The same for calls whose score pass is the first pass over X (a separate criterion
    tensor, the stage entry point)."""
    w, ks = C.c_int32(0), C.c_int32(0)
    _check(lib().dart_score_tile_shape_first_read(C.byref(desc), C.byref(w), C.byref(ks)),
           "dart_score_tile_shape_first_read")
    return int(w.value), int(ks.value)


def dart_static_scratch_bytes() -> int:
    return int(lib().dart_static_scratch_bytes())


def dart_device_status_static(desc, *, stream=None) -> int:
    return int(lib().dart_device_status_static(C.byref(desc), _stream(stream)))


def dart_probe_mfma_dot32(A, B, out, *, stream=None):
    """A, B: bf16 [tiles, 16, 32]; out: float32 [tiles, 16, 16] (raw matrix-core sums)."""
    _check(lib().dart_probe_mfma_dot32(_ptr(A), _ptr(B), _ptr(out), A.shape[0], _stream(stream)),
           "dart_probe_mfma_dot32")


def dart_reduce_profiled(desc, X, Y, keep, ws, events, *, crit=None, crit_D=0, crit_ld=0,
                         pos=None, pos_out=None, cu_keep=None, piv_out=None, S_out=None,
                         stream=None):
    """events: 12 raw hipEvent_t handles (ints): begin and end of the six stages."""
    assert len(events) == 12
    arr = (C.c_void_p * 12)(*[C.c_void_p(int(e)) for e in events])
    _check(lib().dart_reduce_profiled(C.byref(desc), _ptr(X), _ptr(crit), crit_D, crit_ld,
                                      _ptr(pos), _ptr(Y), _ptr(pos_out), _ptr(keep),
                                      _ptr(cu_keep), _ptr(piv_out), _ptr(S_out), _ptr(ws),
                                      ws.numel(), _stream(stream), arr), "dart_reduce_profiled")


def dart_device_status(desc, ws, *, stream=None) -> int:
    return int(lib().dart_device_status(C.byref(desc), _ptr(ws), _stream(stream)))
