"""Thin ctypes binding of the C ABI in include/ap.h (same names, argument marshalling only).

PyTorch supplies device memory and the HIP stream; every step of the computation runs in the
library's own kernels.  There is no fallback: if the shared library has not been built, the
first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# AP_LIBRARY_PATH selects another build of the same library (e.g. one compiled with other flags)
LIB_PATH = os.environ.get("AP_LIBRARY_PATH") or os.path.join(_PKG, "libap_mi355x.so")

AP_OK = 0
AP_ERR_INVALID_ARG = -1
AP_ERR_UNSUPPORTED = -2
AP_ERR_CAPACITY = -3
AP_ERR_HIP = -4
AP_F32 = 0
AP_BF16 = 1

SYMBOLS = ("ap_status_string", "ap_layout_max_tiles", "ap_layout_workspace_bytes",
           "ap_build_layout", "ap_build_layout_cropped", "ap_build_layout_from_map", "ap_build_schedule", "ap_sparse_attn_fwd", "ap_sparse_attn_fwd_cropped",
           "ap_sparse_attn_entmax15_fwd", "ap_fwd_split_workspace_bytes", "ap_sparse_attn_fwd_split",
           "ap_sparse_attn_fwd_split_static", "ap_sparse_attn_decode",
           "ap_build_layout_transpose", "ap_bwd_workspace_bytes", "ap_sparse_attn_bwd",
           "ap_build_col_schedule", "ap_sparse_attn_bwd_sched",
           "ap_entmax15_bwd_workspace_bytes", "ap_sparse_attn_entmax15_bwd",
           "ap_attention_maps_workspace_bytes", "ap_accumulate_attention_maps",
           "ap_accumulate_attention_maps_lse",
           "ap_prune_mask_workspace_bytes", "ap_prune_mask")


class _CSchedule(ctypes.Structure):
    """struct ap_schedule: four device pointers."""
    _fields_ = [("cnt", ctypes.c_void_p), ("start", ctypes.c_void_p), ("cols", ctypes.c_void_p),
                ("bitmaps", ctypes.c_void_p)]


_lib = None


class ApError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, ap_status_string(status), status))


def lib() -> ctypes.CDLL:
    """Load libap_mi355x.so (built by ``python -m paper_2012_02030_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "HIP library %s is missing: build it with `python -m paper_2012_02030_amd.build` "
                "(there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.ap_status_string.restype = ctypes.c_char_p
        L.ap_status_string.argtypes = [i32]
        L.ap_layout_max_tiles.restype = i64
        L.ap_layout_max_tiles.argtypes = [i32] * 5
        L.ap_layout_workspace_bytes.restype = ctypes.c_size_t
        L.ap_layout_workspace_bytes.argtypes = [i32] * 5
        L.ap_build_layout.restype = i32
        L.ap_build_layout.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp,
                                      ctypes.c_size_t, vp]
        L.ap_build_layout_cropped.restype = i32
        L.ap_build_layout_cropped.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp,
                                              ctypes.c_size_t, vp]
        L.ap_build_layout_from_map.restype = i32
        L.ap_build_layout_from_map.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp,
                                               ctypes.c_size_t, vp]
        L.ap_build_schedule.restype = i32
        L.ap_build_schedule.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i64, i32, i32,
                                        ctypes.POINTER(_CSchedule), vp]
        L.ap_sparse_attn_fwd.restype = i32
        L.ap_sparse_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                         ctypes.POINTER(i64), ctypes.POINTER(i64),
                                         ctypes.POINTER(i64), ctypes.POINTER(i64),
                                         vp, vp, vp, i32, i32, ctypes.POINTER(_CSchedule), i32,
                                         ctypes.c_float, vp]
        L.ap_sparse_attn_fwd_cropped.restype = i32
        L.ap_sparse_attn_fwd_cropped.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                                 ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                 ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                 vp, vp, vp, i32, i32, i32, i32, ctypes.POINTER(_CSchedule), i32,
                                                 ctypes.c_float, vp]
        L.ap_sparse_attn_decode.restype = i32
        L.ap_sparse_attn_decode.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                            ctypes.POINTER(i64), ctypes.POINTER(i64),
                                            ctypes.POINTER(i64), ctypes.POINTER(i64),
                                            vp, vp, vp, i32, i32, i32, ctypes.c_float, i32, vp,
                                            ctypes.c_size_t, vp]
        L.ap_sparse_attn_entmax15_fwd.restype = i32
        L.ap_sparse_attn_entmax15_fwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                                  ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                  ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                  vp, vp, vp, i32, i32, ctypes.POINTER(_CSchedule), i32,
                                                  ctypes.c_float, vp]
        L.ap_fwd_split_workspace_bytes.restype = ctypes.c_size_t
        L.ap_fwd_split_workspace_bytes.argtypes = [i32] * 5
        L.ap_sparse_attn_fwd_split.restype = i32
        L.ap_sparse_attn_fwd_split.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                               ctypes.POINTER(i64), ctypes.POINTER(i64),
                                               ctypes.POINTER(i64), ctypes.POINTER(i64),
                                               vp, vp, vp, i32, i32, ctypes.POINTER(_CSchedule), i32,
                                               ctypes.c_float, i32, vp, ctypes.c_size_t, vp]
        L.ap_sparse_attn_fwd_split_static.restype = i32
        L.ap_sparse_attn_fwd_split_static.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                                      ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                      ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                      vp, vp, vp, i32, i32, ctypes.POINTER(_CSchedule), i32,
                                                      ctypes.c_float, i32, vp]
        L.ap_build_layout_transpose.restype = i32
        L.ap_build_layout_transpose.argtypes = [vp, vp, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
        L.ap_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.ap_bwd_workspace_bytes.argtypes = [i32] * 3
        L.ap_sparse_attn_bwd.restype = i32
        L.ap_sparse_attn_bwd.argtypes = [vp] * 9 + [i32] * 6 + [ctypes.POINTER(i64)] * 4 + [vp] * 6 + \
                                        [i32, i32, i32, ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.ap_build_col_schedule.restype = i32
        L.ap_build_col_schedule.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i64, i32, i32,
                                            ctypes.POINTER(_CSchedule), vp]
        L.ap_sparse_attn_bwd_sched.restype = i32
        L.ap_sparse_attn_bwd_sched.argtypes = [vp] * 9 + [i32] * 6 + [ctypes.POINTER(i64)] * 4 + [vp] * 6 + \
                                              [i32, i32, ctypes.POINTER(_CSchedule), ctypes.POINTER(_CSchedule),
                                               i32, ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.ap_entmax15_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.ap_entmax15_bwd_workspace_bytes.argtypes = [i32] * 3
        L.ap_sparse_attn_entmax15_bwd.restype = i32
        L.ap_sparse_attn_entmax15_bwd.argtypes = [vp] * 8 + [i32] * 6 + [ctypes.POINTER(i64)] * 4 + [vp] * 6 + \
                                                 [i32, i32, ctypes.POINTER(_CSchedule), ctypes.POINTER(_CSchedule),
                                                  i32, ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.ap_attention_maps_workspace_bytes.restype = ctypes.c_size_t
        L.ap_attention_maps_workspace_bytes.argtypes = [i32] * 3
        L.ap_accumulate_attention_maps.restype = i32
        L.ap_accumulate_attention_maps.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32,
                                                   ctypes.POINTER(i64), ctypes.POINTER(i64), i32,
                                                   ctypes.c_float, ctypes.c_float, vp, vp,
                                                   ctypes.c_size_t, vp]
        L.ap_accumulate_attention_maps_lse.restype = i32
        L.ap_accumulate_attention_maps_lse.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                                       ctypes.POINTER(i64), ctypes.POINTER(i64), i32,
                                                       ctypes.c_float, ctypes.c_float, vp, vp,
                                                       ctypes.c_size_t, vp]
        L.ap_prune_mask_workspace_bytes.restype = ctypes.c_size_t
        L.ap_prune_mask_workspace_bytes.argtypes = []
        L.ap_prune_mask.restype = i32
        L.ap_prune_mask.argtypes = [vp, i32, i32, i32, i32, ctypes.c_double, vp, vp, vp,
                                    ctypes.c_size_t, vp]
        _lib = L
    return _lib


def ap_status_string(status: int) -> str:
    return lib().ap_status_string(int(status)).decode()


def ap_layout_max_tiles(H: int, Lq: int, Lk: int, block_m: int, block_n: int) -> int:
    return int(lib().ap_layout_max_tiles(H, Lq, Lk, block_m, block_n))


def ap_layout_workspace_bytes(H: int, Lq: int, Lk: int, block_m: int, block_n: int) -> int:
    return int(lib().ap_layout_workspace_bytes(H, Lq, Lk, block_m, block_n))


class Layout(NamedTuple):
    """Device arrays of a block-sparse layout plus the sizes it was built for."""
    row_ptr: torch.Tensor    # int32 [H*nQB + 1]
    col_idx: torch.Tensor    # int32 [cap]
    bitmaps: torch.Tensor    # int64 storage of uint64 words [cap, block_m, ceil(block_n/64)]
    nnz: torch.Tensor        # int64 [1] on device
    H: int
    Lq: int
    Lk: int
    block_m: int
    block_n: int


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def ap_build_layout(mask: torch.Tensor, block_m: int = 64, block_n: int = 64,
                    cap: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None,
                    count_only: bool = False, crop: Optional[tuple] = None) -> Layout:
    """mask: uint8/bool device tensor [H, Lq, Lk], nonzero = kept.  Asynchronous on the stream.

    crop = (Lq', Lk') builds the layout of the mask's top-left corner (ap_build_layout_cropped)."""
    if mask.dtype == torch.bool:
        mask = mask.view(torch.uint8)
    if mask.dtype != torch.uint8 or mask.dim() != 3 or not mask.is_cuda:
        raise ValueError("mask must be a uint8/bool device tensor [H, Lq, Lk]")
    mask = mask.contiguous()
    H, Lq_stored, Lk_stored = mask.shape
    Lq, Lk = (Lq_stored, Lk_stored) if crop is None else (int(crop[0]), int(crop[1]))
    max_tiles = ap_layout_max_tiles(H, Lq, Lk, block_m, block_n)
    if max_tiles < 0:
        raise ApError(AP_ERR_UNSUPPORTED, "ap_layout_max_tiles")
    if cap is None:
        cap = max_tiles
    dev = mask.device
    nqb = -(-Lq // block_m)
    W = -(-block_n // 64)
    row_ptr = torch.empty(H * nqb + 1, dtype=torch.int32, device=dev)
    nnz = torch.empty(1, dtype=torch.int64, device=dev)
    ws_bytes = ap_layout_workspace_bytes(H, Lq, Lk, block_m, block_n)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    if count_only:
        col_idx = torch.empty(0, dtype=torch.int32, device=dev)
        bitmaps = torch.empty((0, block_m, W), dtype=torch.int64, device=dev)
        cptr = bptr = None
    else:
        col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
        bitmaps = torch.empty((max(cap, 1), block_m, W), dtype=torch.int64, device=dev)
        cptr, bptr = col_idx.data_ptr(), bitmaps.data_ptr()
    if crop is None:
        st = lib().ap_build_layout(mask.data_ptr(), H, Lq, Lk, block_m, block_n, row_ptr.data_ptr(),
                                   cptr, bptr, cap, nnz.data_ptr(), ws.data_ptr(), ws_bytes,
                                   _stream_ptr(stream))
    else:
        st = lib().ap_build_layout_cropped(mask.data_ptr(), H, Lq_stored, Lk_stored, Lq, Lk, block_m, block_n,
                                           row_ptr.data_ptr(), cptr, bptr, cap, nnz.data_ptr(),
                                           ws.data_ptr(), ws_bytes, _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_build_layout")
    # ws is released to torch's caching allocator here; the allocator is stream-ordered, so the
    # kernels enqueued above finish with it before any later allocation on this stream reuses it
    return Layout(row_ptr, col_idx, bitmaps, nnz, H, Lq, Lk, block_m, block_n)


def ap_build_layout_from_map(abar: torch.Tensor, tau: torch.Tensor, causal: bool = False, block_m: int = 64,
                             block_n: int = 64, cap: Optional[int] = None,
                             stream: Optional[torch.cuda.Stream] = None) -> Layout:
    """Layout of the mask {not (abar < tau), and visible if causal} without writing that mask.

    abar: float32 device tensor [H, Lq, Lk]; tau: float32 device tensor with one element (e.g. the
    second result of ap_prune_mask).  Asynchronous on the stream."""
    if abar.dtype != torch.float32 or abar.dim() != 3 or not abar.is_cuda:
        raise ValueError("abar must be a float32 device tensor [H, Lq, Lk]")
    if tau.dtype != torch.float32 or tau.numel() != 1 or tau.device != abar.device:
        raise ValueError("tau must be a float32 tensor with one element on abar's device")
    abar = abar.contiguous()
    H, Lq, Lk = abar.shape
    max_tiles = ap_layout_max_tiles(H, Lq, Lk, block_m, block_n)
    if max_tiles < 0:
        raise ApError(AP_ERR_UNSUPPORTED, "ap_layout_max_tiles")
    if cap is None:
        cap = max_tiles
    dev = abar.device
    nqb = -(-Lq // block_m)
    W = -(-block_n // 64)
    row_ptr = torch.empty(H * nqb + 1, dtype=torch.int32, device=dev)
    nnz = torch.empty(1, dtype=torch.int64, device=dev)
    ws_bytes = ap_layout_workspace_bytes(H, Lq, Lk, block_m, block_n)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    bitmaps = torch.empty((max(cap, 1), block_m, W), dtype=torch.int64, device=dev)
    st = lib().ap_build_layout_from_map(abar.data_ptr(), tau.data_ptr(), H, Lq, Lk, int(bool(causal)), block_m,
                                        block_n, row_ptr.data_ptr(), col_idx.data_ptr(), bitmaps.data_ptr(), cap,
                                        nnz.data_ptr(), ws.data_ptr(), ws_bytes, _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_build_layout_from_map")
    return Layout(row_ptr, col_idx, bitmaps, nnz, H, Lq, Lk, block_m, block_n)


class Schedule(NamedTuple):
    """Device arrays of a visit schedule (see ap_schedule in include/ap.h)."""
    cnt: torch.Tensor        # int32 [H*nQB]
    start: torch.Tensor      # int32 [cap]
    cols: torch.Tensor       # int32 [cap, 64]
    bitmaps: torch.Tensor    # int64 storage of uint64 words [cap, block_m]
    causal: bool
    min_cols: int

    def c_struct(self) -> _CSchedule:
        return _CSchedule(self.cnt.data_ptr(), self.start.data_ptr(), self.cols.data_ptr(),
                          self.bitmaps.data_ptr())


def ap_build_schedule(layout: Layout, causal: bool = False, min_cols: int = 0,
                      stream: Optional[torch.cuda.Stream] = None) -> Schedule:
    """Derive the visit schedule of a layout (block_n = 64).  Asynchronous on the stream."""
    dev = layout.row_ptr.device
    cap = int(layout.col_idx.shape[0])
    nrows = int(layout.row_ptr.shape[0]) - 1
    sched = Schedule(torch.empty(nrows, dtype=torch.int32, device=dev),
                     torch.empty(cap, dtype=torch.int32, device=dev),
                     torch.empty((cap, 64), dtype=torch.int32, device=dev),
                     torch.empty((cap, layout.block_m), dtype=torch.int64, device=dev),
                     bool(causal), int(min_cols))
    cs = sched.c_struct()
    st = lib().ap_build_schedule(layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(),
                                 layout.bitmaps.data_ptr(), layout.H, layout.Lq, layout.Lk,
                                 layout.block_m, layout.block_n, cap, int(bool(causal)), int(min_cols),
                                 ctypes.byref(cs), _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_build_schedule")
    return sched


def _check_out(out: torch.Tensor, like: torch.Tensor, name: str = "out"):
    """A caller-supplied output must be what the kernels will write: like's shape, dtype and
    device, last dimension contiguous (the C ABI sees only a pointer and three strides)."""
    if tuple(out.shape) != tuple(like.shape) or out.dtype != like.dtype or out.device != like.device:
        raise ValueError("%s must be a %s tensor of shape %s on %s" % (
            name, like.dtype, tuple(like.shape), like.device))
    if out.stride(3) != 1:
        raise ValueError("%s: last dimension must be contiguous" % name)


def _check_rows_f32(t: torch.Tensor, like: torch.Tensor, name: str):
    """Per-query statistics (lse, tau): contiguous float32 [B, H, Lq] on like's device."""
    if t.dtype != torch.float32 or tuple(t.shape) != tuple(like.shape[:3]) or t.device != like.device \
            or not t.is_contiguous():
        raise ValueError("%s must be a contiguous float32 tensor of shape %s on %s" % (
            name, tuple(like.shape[:3]), like.device))


def _strides3(t: torch.Tensor):
    return (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def ap_sparse_attn_fwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, layout: Layout,
                       causal: bool = False, softmax_scale: float = 0.0,
                       out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                       return_lse: bool = True, stream: Optional[torch.cuda.Stream] = None,
                       sched: Optional[Schedule] = None, crop: bool = False):
    """Q [B,H,Lq,D], K/V [B,H,Lk,D] device tensors (fp32 or bf16, last dim contiguous).

    crop=True: Lq, Lk may be smaller than the sizes the layout was built for; the call then runs
    under the top-left corner of that mask (ap_sparse_attn_fwd_cropped).
    Returns (O, lse); lse is None when return_lse is False.  Asynchronous on the stream.
    """
    if Q.dtype == torch.bfloat16:
        dt = AP_BF16
    elif Q.dtype == torch.float32:
        dt = AP_F32
    else:
        raise ValueError("dtype must be float32 or bfloat16")
    if K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must share a dtype")
    if Q.dim() != 4 or K.dim() != 4 or V.dim() != 4:
        raise ValueError("Q, K, V must be [B, H, L, D]")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D):
        raise ValueError("K/V shape mismatch")
    cropped = (Lq, Lk) != (layout.Lq, layout.Lk)
    if H != layout.H or Lq > layout.Lq or Lk > layout.Lk or (cropped and not crop):
        raise ValueError("layout was built for other sizes")
    for t in (Q, K, V):
        if t.stride(3) != 1:
            raise ValueError("last dimension must be contiguous")
    if sched is not None and sched.causal != bool(causal):
        raise ValueError("schedule was built with causal=%s" % sched.causal)
    cs = sched.c_struct() if sched is not None else None
    if out is None:
        out = torch.empty((B, H, Lq, D), dtype=Q.dtype, device=Q.device)
    else:
        _check_out(out, Q)
    if lse is None and return_lse:
        lse = torch.empty((B, H, Lq), dtype=torch.float32, device=Q.device)
    elif lse is not None:
        _check_rows_f32(lse, Q, "lse")
    head = (Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
            lse.data_ptr() if lse is not None else None, dt, B, H, Lq, Lk, D,
            _strides3(Q), _strides3(K), _strides3(V), _strides3(out),
            layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
            layout.block_m, layout.block_n)
    tail = (ctypes.byref(cs) if cs is not None else None, int(bool(causal)), float(softmax_scale),
            _stream_ptr(stream))
    if crop:
        st = lib().ap_sparse_attn_fwd_cropped(*head, layout.Lq, layout.Lk, *tail)
    else:
        st = lib().ap_sparse_attn_fwd(*head, *tail)
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_fwd")
    return out, lse


def ap_sparse_attn_decode(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, layout: Layout,
                          causal: bool = False, softmax_scale: float = 0.0,
                          out: Optional[torch.Tensor] = None, return_lse: bool = True,
                          stream: Optional[torch.cuda.Stream] = None, splits: int = 1):
    """ap_sparse_attn_fwd for one or a few queries against many keys (bf16), `splits` workgroups
    per query.  Returns (O, lse)."""
    if Q.dtype != torch.bfloat16 or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must be bfloat16")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D):
        raise ValueError("K/V shape mismatch")
    if (H, Lq, Lk) != (layout.H, layout.Lq, layout.Lk):
        raise ValueError("layout was built for other sizes")
    for t in (Q, K, V):
        if t.stride(3) != 1:
            raise ValueError("last dimension must be contiguous")
    if out is None:
        out = torch.empty((B, H, Lq, D), dtype=Q.dtype, device=Q.device)
    else:
        _check_out(out, Q)
    lse = torch.empty((B, H, Lq), dtype=torch.float32, device=Q.device) if return_lse else None
    ws_bytes = ap_fwd_split_workspace_bytes(B, H, Lq, D, splits) if splits > 1 else 0
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=Q.device)
    st = lib().ap_sparse_attn_decode(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
        lse.data_ptr() if lse is not None else None, AP_BF16, B, H, Lq, Lk, D,
        _strides3(Q), _strides3(K), _strides3(V), _strides3(out),
        layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
        layout.block_m, layout.block_n, int(bool(causal)), float(softmax_scale), int(splits),
        ws.data_ptr(), ws_bytes, _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_decode")
    return out, lse


def ap_sparse_attn_entmax15_fwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, layout: Layout,
                                causal: bool = False, softmax_scale: float = 0.0,
                                out: Optional[torch.Tensor] = None, return_tau: bool = True,
                                stream: Optional[torch.cuda.Stream] = None,
                                sched: Optional[Schedule] = None):
    """Masked attention with the 1.5-entmax normaliser (bf16, block_m 64).  Returns (O, tau)."""
    if sched is not None and sched.causal != bool(causal):
        raise ValueError("schedule was built with causal=%s" % sched.causal)
    cs = sched.c_struct() if sched is not None else None
    if Q.dtype != torch.bfloat16 or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must be bfloat16")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D):
        raise ValueError("K/V shape mismatch")
    if (H, Lq, Lk) != (layout.H, layout.Lq, layout.Lk):
        raise ValueError("layout was built for other sizes")
    if out is None:
        out = torch.empty((B, H, Lq, D), dtype=Q.dtype, device=Q.device)
    else:
        _check_out(out, Q)
    tau = torch.empty((B, H, Lq), dtype=torch.float32, device=Q.device) if return_tau else None
    st = lib().ap_sparse_attn_entmax15_fwd(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
        tau.data_ptr() if tau is not None else None, AP_BF16, B, H, Lq, Lk, D,
        _strides3(Q), _strides3(K), _strides3(V), _strides3(out),
        layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
        layout.block_m, layout.block_n, ctypes.byref(cs) if cs is not None else None,
        int(bool(causal)), float(softmax_scale), _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_entmax15_fwd")
    return out, tau


def ap_fwd_split_workspace_bytes(B: int, H: int, Lq: int, D: int, splits: int) -> int:
    return int(lib().ap_fwd_split_workspace_bytes(B, H, Lq, D, splits))


def ap_sparse_attn_fwd_split(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, layout: Layout,
                             splits: int, causal: bool = False, softmax_scale: float = 0.0,
                             out: Optional[torch.Tensor] = None, return_lse: bool = True,
                             stream: Optional[torch.cuda.Stream] = None,
                             sched: Optional[Schedule] = None):
    """ap_sparse_attn_fwd with the entries of every block row cut into `splits` chunks (bf16,
    block_m 64): for few queries against many keys.  Returns (O, lse).  Asynchronous."""
    if Q.dtype != torch.bfloat16 or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must be bfloat16")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D):
        raise ValueError("K/V shape mismatch")
    if (H, Lq, Lk) != (layout.H, layout.Lq, layout.Lk):
        raise ValueError("layout was built for other sizes")
    if sched is not None and sched.causal != bool(causal):
        raise ValueError("schedule was built with causal=%s" % sched.causal)
    cs = sched.c_struct() if sched is not None else None
    if out is None:
        out = torch.empty((B, H, Lq, D), dtype=Q.dtype, device=Q.device)
    else:
        _check_out(out, Q)
    lse = torch.empty((B, H, Lq), dtype=torch.float32, device=Q.device) if return_lse else None
    ws_bytes = ap_fwd_split_workspace_bytes(B, H, Lq, D, splits)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=Q.device)
    st = lib().ap_sparse_attn_fwd_split(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
        lse.data_ptr() if lse is not None else None, AP_BF16, B, H, Lq, Lk, D,
        _strides3(Q), _strides3(K), _strides3(V), _strides3(out),
        layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
        layout.block_m, layout.block_n, ctypes.byref(cs) if cs is not None else None,
        int(bool(causal)), float(softmax_scale), int(splits), ws.data_ptr(), ws_bytes,
        _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_fwd_split")
    return out, lse


AP_FWD_SPLIT_STATIC_MAX_BYTES = 32 << 20


def ap_sparse_attn_fwd_split_static(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, layout: Layout,
                                    splits: int, out: torch.Tensor, lse: Optional[torch.Tensor] = None,
                                    causal: bool = False, softmax_scale: float = 0.0,
                                    stream: Optional[torch.cuda.Stream] = None,
                                    sched: Optional[Schedule] = None):
    """ap_sparse_attn_fwd_split without a workspace: the partial results live in the library's own
    device array.  Nothing is allocated here either, so the caller passes `out` (and `lse`, or
    None to skip it).  Calls that may overlap on one GPU race; serialise them."""
    if Q.dtype != torch.bfloat16 or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must be bfloat16")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D):
        raise ValueError("K/V shape mismatch")
    if (H, Lq, Lk) != (layout.H, layout.Lq, layout.Lk):
        raise ValueError("layout was built for other sizes")
    if sched is not None and sched.causal != bool(causal):
        raise ValueError("schedule was built with causal=%s" % sched.causal)
    _check_out(out, Q)
    if lse is not None:
        _check_rows_f32(lse, Q, "lse")
    cs = sched.c_struct() if sched is not None else None
    st = lib().ap_sparse_attn_fwd_split_static(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
        lse.data_ptr() if lse is not None else None, AP_BF16, B, H, Lq, Lk, D,
        _strides3(Q), _strides3(K), _strides3(V), _strides3(out),
        layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
        layout.block_m, layout.block_n, ctypes.byref(cs) if cs is not None else None,
        int(bool(causal)), float(softmax_scale), int(splits), _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_fwd_split_static")
    return out, lse


class LayoutT(NamedTuple):
    """Transpose of a layout: the tiles of every (head, block column), ascending block rows."""
    col_ptr: torch.Tensor    # int32 [H*nKB + 1]
    row_idx: torch.Tensor    # int32 [cap]
    tile_idx: torch.Tensor   # int32 [cap]


def ap_build_layout_transpose(layout: Layout, stream: Optional[torch.cuda.Stream] = None) -> LayoutT:
    """Asynchronous on the stream; the layout must not be truncated."""
    dev = layout.row_ptr.device
    cap = int(layout.col_idx.shape[0])
    nkb = -(-layout.Lk // layout.block_n)
    lt = LayoutT(torch.empty(layout.H * nkb + 1, dtype=torch.int32, device=dev),
                 torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
                 torch.empty(max(cap, 1), dtype=torch.int32, device=dev))
    st = lib().ap_build_layout_transpose(layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.H,
                                         layout.Lq, layout.Lk, layout.block_m, layout.block_n, cap,
                                         lt.col_ptr.data_ptr(), lt.row_idx.data_ptr(),
                                         lt.tile_idx.data_ptr(), _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_build_layout_transpose")
    return lt


def ap_bwd_workspace_bytes(B: int, H: int, Lq: int) -> int:
    return int(lib().ap_bwd_workspace_bytes(B, H, Lq))


def ap_build_col_schedule(layout: Layout, layout_t: LayoutT, causal: bool = False, min_rows: int = 0,
                          stream: Optional[torch.cuda.Stream] = None) -> Schedule:
    """Derive the column schedule (for dK, dV) from a layout and its transpose.  Asynchronous."""
    dev = layout.row_ptr.device
    cap = int(layout.col_idx.shape[0])
    ncols = int(layout_t.col_ptr.shape[0]) - 1
    sched = Schedule(torch.empty(2 * ncols + layout.H, dtype=torch.int32, device=dev),
                     torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
                     torch.empty((max(cap, 1), 64), dtype=torch.int32, device=dev),
                     torch.empty((max(cap, 1), 64), dtype=torch.int64, device=dev),
                     bool(causal), int(min_rows))
    cs = sched.c_struct()
    st = lib().ap_build_col_schedule(layout_t.col_ptr.data_ptr(), layout_t.row_idx.data_ptr(),
                                     layout_t.tile_idx.data_ptr(), layout.bitmaps.data_ptr(), layout.H,
                                     layout.Lq, layout.Lk, layout.block_m, layout.block_n, cap,
                                     int(bool(causal)), int(min_rows), ctypes.byref(cs), _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_build_col_schedule")
    return sched


def ap_sparse_attn_bwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, O: torch.Tensor,
                       dO: torch.Tensor, lse: torch.Tensor, layout: Layout, layout_t: LayoutT,
                       causal: bool = False, softmax_scale: float = 0.0,
                       stream: Optional[torch.cuda.Stream] = None,
                       sched: Optional[Schedule] = None, col_sched: Optional[Schedule] = None):
    """Gradients (dQ, dK, dV) of ap_sparse_attn_fwd's O with respect to Q, K, V (bf16).

    O and lse are the forward call's outputs; dO must have O's strides.  With a row schedule
    and/or a column schedule the call goes to ap_sparse_attn_bwd_sched.  Asynchronous on the stream."""
    for sc in (sched, col_sched):
        if sc is not None and sc.causal != bool(causal):
            raise ValueError("schedule was built with another `causal`")
    for t in (Q, K, V, O, dO):
        if t.dtype != torch.bfloat16 or t.dim() != 4 or t.stride(3) != 1:
            raise ValueError("Q, K, V, O, dO must be bfloat16 [B, H, L, D] with a contiguous last dimension")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D) or \
            tuple(O.shape) != (B, H, Lq, D) or tuple(dO.shape) != (B, H, Lq, D):
        raise ValueError("shape mismatch")
    if (H, Lq, Lk) != (layout.H, layout.Lq, layout.Lk):
        raise ValueError("layout was built for other sizes")
    if dO.stride() != O.stride():
        dO = dO.contiguous() if O.is_contiguous() else dO.clone(memory_format=torch.preserve_format)
        if dO.stride() != O.stride():
            raise ValueError("dO must have O's strides")
    lse = lse.contiguous()
    _check_rows_f32(lse, Q, "lse")
    dQ = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    dK = torch.empty_strided(K.shape, K.stride(), dtype=K.dtype, device=K.device)
    dV = torch.empty_strided(V.shape, V.stride(), dtype=V.dtype, device=V.device)
    ws_bytes = ap_bwd_workspace_bytes(B, H, Lq)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=Q.device)
    head = (Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), lse.data_ptr(),
            dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), AP_BF16, B, H, Lq, Lk, D,
            _strides3(Q), _strides3(K), _strides3(V), _strides3(O),
            layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
            layout_t.col_ptr.data_ptr(), layout_t.row_idx.data_ptr(), layout_t.tile_idx.data_ptr(),
            layout.block_m, layout.block_n)
    tail = (int(bool(causal)), float(softmax_scale), ws.data_ptr(), ws_bytes, _stream_ptr(stream))
    if sched is None and col_sched is None:
        st = lib().ap_sparse_attn_bwd(*head, *tail)
    else:
        cs = sched.c_struct() if sched is not None else None
        ccs = col_sched.c_struct() if col_sched is not None else None
        st = lib().ap_sparse_attn_bwd_sched(*head, ctypes.byref(cs) if cs is not None else None,
                                            ctypes.byref(ccs) if ccs is not None else None, *tail)
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_bwd")
    return dQ, dK, dV


def ap_entmax15_bwd_workspace_bytes(B: int, H: int, Lq: int) -> int:
    return int(lib().ap_entmax15_bwd_workspace_bytes(B, H, Lq))


def ap_sparse_attn_entmax15_bwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, dO: torch.Tensor,
                                tau: torch.Tensor, layout: Layout, layout_t: LayoutT, sched: Schedule,
                                col_sched: Schedule, causal: bool = False, softmax_scale: float = 0.0,
                                stream: Optional[torch.cuda.Stream] = None):
    """Gradients (dQ, dK, dV) of ap_sparse_attn_entmax15_fwd's O with respect to Q, K, V (bf16).

    tau is the forward call's second output; both schedules are required.  Asynchronous on the stream."""
    for t in (Q, K, V, dO):
        if t.dtype != torch.bfloat16 or t.dim() != 4 or t.stride(3) != 1:
            raise ValueError("Q, K, V, dO must be bfloat16 [B, H, L, D] with a contiguous last dimension")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D) or tuple(V.shape) != (B, H, Lk, D) or tuple(dO.shape) != (B, H, Lq, D):
        raise ValueError("shape mismatch")
    if (H, Lq, Lk) != (layout.H, layout.Lq, layout.Lk):
        raise ValueError("layout was built for other sizes")
    for sc in (sched, col_sched):
        if sc.causal != bool(causal):
            raise ValueError("schedule was built with another `causal`")
    tau = tau.contiguous()
    _check_rows_f32(tau, Q, "tau")
    dQ = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    dK = torch.empty_strided(K.shape, K.stride(), dtype=K.dtype, device=K.device)
    dV = torch.empty_strided(V.shape, V.stride(), dtype=V.dtype, device=V.device)
    ws_bytes = ap_entmax15_bwd_workspace_bytes(B, H, Lq)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=Q.device)
    cs, ccs = sched.c_struct(), col_sched.c_struct()
    st = lib().ap_sparse_attn_entmax15_bwd(
        Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(), tau.data_ptr(),
        dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), AP_BF16, B, H, Lq, Lk, D,
        _strides3(Q), _strides3(K), _strides3(V), _strides3(dO),
        layout.row_ptr.data_ptr(), layout.col_idx.data_ptr(), layout.bitmaps.data_ptr(),
        layout_t.col_ptr.data_ptr(), layout_t.row_idx.data_ptr(), layout_t.tile_idx.data_ptr(),
        layout.block_m, layout.block_n, ctypes.byref(cs), ctypes.byref(ccs), int(bool(causal)),
        float(softmax_scale), ws.data_ptr(), ws_bytes, _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_sparse_attn_entmax15_bwd")
    return dQ, dK, dV


def ap_attention_maps_workspace_bytes(B: int, H: int, Lq: int) -> int:
    return int(lib().ap_attention_maps_workspace_bytes(B, H, Lq))


def ap_accumulate_attention_maps(Q: torch.Tensor, K: torch.Tensor,
                                 abar: Optional[torch.Tensor] = None, causal: bool = False,
                                 softmax_scale: float = 0.0, weight: float = 1.0,
                                 stream: Optional[torch.cuda.Stream] = None,
                                 lse: Optional[torch.Tensor] = None) -> torch.Tensor:
    """abar [H,Lq,Lk] fp32 += weight * sum_b softmax(Q_b K_b^T * scale); a new zeroed abar when
    none is given.  Q [B,H,Lq,D], K [B,H,Lk,D] bf16 device tensors.  lse: the log-sum-exp
    [B,H,Lq] of the unpruned attention call on the same inputs, if it is at hand
    (ap_accumulate_attention_maps_lse).  Asynchronous on the stream."""
    if Q.dtype != torch.bfloat16 or K.dtype != torch.bfloat16:
        raise ValueError("Q and K must be bfloat16")
    if Q.dim() != 4 or K.dim() != 4:
        raise ValueError("Q, K must be [B, H, L, D]")
    B, H, Lq, D = Q.shape
    Lk = K.shape[2]
    if tuple(K.shape) != (B, H, Lk, D):
        raise ValueError("K shape mismatch")
    if Q.stride(3) != 1 or K.stride(3) != 1:
        raise ValueError("last dimension must be contiguous")
    if abar is None:
        abar = torch.zeros((H, Lq, Lk), dtype=torch.float32, device=Q.device)
    if abar.dtype != torch.float32 or tuple(abar.shape) != (H, Lq, Lk) or not abar.is_contiguous():
        raise ValueError("abar must be a contiguous float32 tensor [H, Lq, Lk]")
    ws_bytes = ap_attention_maps_workspace_bytes(B, H, Lq)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=Q.device)
    tail = (AP_BF16, B, H, Lq, Lk, D, _strides3(Q), _strides3(K), int(bool(causal)), float(softmax_scale),
            float(weight), abar.data_ptr(), ws.data_ptr(), ws_bytes, _stream_ptr(stream))
    if lse is None:
        st = lib().ap_accumulate_attention_maps(Q.data_ptr(), K.data_ptr(), *tail)
    else:
        if lse.dtype != torch.float32 or tuple(lse.shape) != (B, H, Lq):
            raise ValueError("lse must be float32 [B, H, Lq]")
        lse = lse.contiguous()
        st = lib().ap_accumulate_attention_maps_lse(Q.data_ptr(), K.data_ptr(), lse.data_ptr(), *tail)
    if st != AP_OK:
        raise ApError(st, "ap_accumulate_attention_maps")
    return abar


def ap_prune_mask_workspace_bytes() -> int:
    return int(lib().ap_prune_mask_workspace_bytes())


def ap_prune_mask(abar: torch.Tensor, prune_fraction: float, causal: bool = False,
                  stream: Optional[torch.cuda.Stream] = None, threshold_only: bool = False):
    """abar: float32 device tensor [H, Lq, Lk], the mean maps of all heads of one layer.

    Returns (mask uint8 [H,Lq,Lk] with 1 = kept, tau float32 [1] on device); with threshold_only the
    mask is not written and None is returned in its place.  Asynchronous."""
    if abar.dtype != torch.float32 or abar.dim() != 3 or not abar.is_cuda:
        raise ValueError("abar must be a float32 device tensor [H, Lq, Lk]")
    abar = abar.contiguous()
    H, Lq, Lk = abar.shape
    mask = None if threshold_only else torch.empty((H, Lq, Lk), dtype=torch.uint8, device=abar.device)
    tau = torch.empty(1, dtype=torch.float32, device=abar.device)
    ws_bytes = ap_prune_mask_workspace_bytes()
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=abar.device)
    st = lib().ap_prune_mask(abar.data_ptr(), H, Lq, Lk, int(bool(causal)), float(prune_fraction),
                             mask.data_ptr() if mask is not None else None, tau.data_ptr(), ws.data_ptr(), ws_bytes,
                             _stream_ptr(stream))
    if st != AP_OK:
        raise ApError(st, "ap_prune_mask")
    return mask, tau
