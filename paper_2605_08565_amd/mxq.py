"""Thin Python binding over the C ABI of libmxq (include/mxq.h).

Argument marshalling only: every function takes torch tensors that already live on the GPU,
passes their device pointers and the current HIP stream to the library and returns.  Nothing
is computed here and there is no CPU fallback -- a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxq.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_ALIGNMENT, ERR_HIP = 0, -1, -2, -3, -4
ELEM_E2M1 = 0
SCALE_E8M0, SCALE_E4M3, SCALE_UE5M3 = 0, 1, 2
RECIPE_ABSMAX, RECIPE_ABSMAX_PZ, RECIPE_4OVER6, RECIPE_4OVER6_PZ, RECIPE_BRUTE, RECIPE_BRUTE_PRUNED = 0, 1, 2, 3, 4, 5
DT_BF16, DT_F32 = 0, 1

_lib = None


class _Tensor(ctypes.Structure):
    """struct mxq_tensor of include/mxq.h"""
    _fields_ = [("x", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("codes_out", ctypes.c_void_p), ("scales_out", ctypes.c_void_p), ("sse_out", ctypes.c_void_p)]


class MxqError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libmxq: {status_string(status)} ({status})")


def lib() -> ctypes.CDLL:
    """Loads libmxq.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2605_08565_amd.build` (hipcc, gfx950)")
    L = ctypes.CDLL(LIB_PATH)
    i64, i32, f32, vp, u8 = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_uint8
    L.mxq_quantize.restype = i32
    L.mxq_quantize.argtypes = [vp, i64, i64, i32, i32, i32, i32, f32, vp, vp, vp, i32, vp]
    L.mxq_quantize_clip.restype = i32
    L.mxq_quantize_clip.argtypes = [vp, i64, i64, i32, i32, i32, i32, f32, vp, vp, vp, vp, i32, vp]
    L.mxq_quantize_batch.restype = i32
    L.mxq_quantize_batch.argtypes = [ctypes.POINTER(_Tensor), i32, i32, i32, i32, i32, i32, vp]
    L.mxq_quantize_hier.restype = i32
    L.mxq_quantize_hier.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp]
    L.mxq_dequantize.restype = i32
    L.mxq_dequantize.argtypes = [vp, vp, i64, i64, i32, i32, i32, f32, vp, i32, vp]
    L.mxq_dequantize_hier.restype = i32
    L.mxq_dequantize_hier.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp, i32, vp]
    L.mxq_tensor_absmax.restype = i32
    L.mxq_tensor_absmax.argtypes = [vp, i64, i64, i32, vp, vp]
    L.mxq_tensor_absmax_acc.restype = i32
    L.mxq_tensor_absmax_acc.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    L.mxq_tensor_absmax_workspace_size.restype = ctypes.c_size_t
    L.mxq_tensor_absmax_workspace_size.argtypes = []
    L.mxq_tensor_absmax_ws.restype = i32
    L.mxq_tensor_absmax_ws.argtypes = [vp, i64, i64, i32, vp, vp, ctypes.c_size_t, vp]
    L.mxq_tensor_absmax_static.restype = i32
    L.mxq_tensor_absmax_static.argtypes = [vp, i64, i64, i32, vp, vp]
    L.mxq_clip_sse.restype = i32
    L.mxq_clip_sse.argtypes = [vp, vp, i64, i64, i32, i32, i32, f32, vp, i32, vp]
    L.mxq_histogram.restype = i32
    L.mxq_histogram.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp]
    L.mxq_tensor_scale_from_absmax.restype = f32
    L.mxq_tensor_scale_from_absmax.argtypes = [f32, i32, i32]
    L.mxq_scale_decode.restype = f32
    L.mxq_scale_decode.argtypes = [i32, u8]
    L.mxq_num_candidates.restype = i32
    L.mxq_num_candidates.argtypes = [i32]
    L.mxq_status_string.restype = ctypes.c_char_p
    L.mxq_status_string.argtypes = [i32]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().mxq_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return DT_BF16
    if t.dtype == torch.float32:
        return DT_F32
    raise TypeError("libmxq takes bfloat16 or float32 tensors")


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _check(status: int) -> None:
    if status != OK:
        raise MxqError(status)


def _need(t: torch.Tensor, nbytes: int, name: str, dtype: torch.dtype | None = None) -> None:
    """The library trusts its pointers: refuse a buffer it would read or write past."""
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous tensor on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}")
    if t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{name} holds {t.numel() * t.element_size()} bytes, {nbytes} are needed")


def _nblocks(rows: int, cols: int, block: int) -> int:
    return rows * (cols // block) if block > 0 else 0


def quantize(x: torch.Tensor, block: int, scale_fmt: int, recipe: int, tensor_scale: float = 1.0,
             codes_out: torch.Tensor | None = None, scales_out: torch.Tensor | None = None,
             sse_out: torch.Tensor | None = None, want_sse: bool = True, stream=None,
             elem_fmt: int = ELEM_E2M1, clip_sse_out: torch.Tensor | None = None):
    """mxq_quantize on a 2-D contiguous CUDA tensor. Returns (codes, scales, sse).  With
    `clip_sse_out` (fp32 [rows, cols/block]) mxq_quantize_clip, which also fills that tensor."""
    if not x.is_cuda or x.dim() != 2 or not x.is_contiguous():
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, cols = x.shape
    dev = x.device
    if codes_out is None:
        codes_out = torch.empty((rows, cols // 2), dtype=torch.uint8, device=dev)
    if scales_out is None:
        scales_out = torch.empty((rows, cols // block if block > 0 else 0), dtype=torch.uint8, device=dev)
    if sse_out is None and want_sse:
        sse_out = torch.empty((rows, cols // block if block > 0 else 0), dtype=torch.float32, device=dev)
    _need(codes_out, rows * cols // 2, "codes_out", torch.uint8)
    _need(scales_out, _nblocks(rows, cols, block), "scales_out", torch.uint8)
    if sse_out is not None:
        _need(sse_out, 4 * _nblocks(rows, cols, block), "sse_out", torch.float32)
    if clip_sse_out is not None:
        _need(clip_sse_out, 4 * _nblocks(rows, cols, block), "clip_sse_out", torch.float32)
        _check(lib().mxq_quantize_clip(x.data_ptr(), rows, cols, block, elem_fmt, scale_fmt, recipe,
                                       float(tensor_scale), codes_out.data_ptr(), scales_out.data_ptr(),
                                       sse_out.data_ptr() if sse_out is not None else None,
                                       clip_sse_out.data_ptr(), _dtype_code(x), _stream_ptr(stream)))
        return codes_out, scales_out, sse_out
    _check(lib().mxq_quantize(x.data_ptr(), rows, cols, block, elem_fmt, scale_fmt, recipe,
                              float(tensor_scale), codes_out.data_ptr(), scales_out.data_ptr(),
                              sse_out.data_ptr() if sse_out is not None else None,
                              _dtype_code(x), _stream_ptr(stream)))
    return codes_out, scales_out, sse_out


def quantize_batch(xs, block: int, scale_fmt: int, recipe: int, outs=None, want_sse: bool = True, stream=None,
                   elem_fmt: int = ELEM_E2M1):
    """mxq_quantize_batch: the 2-D contiguous CUDA tensors `xs` (one dtype) in as few launches as
    possible.  `outs`: optional list of (codes, scales, sse-or-None) per tensor.  Returns that list."""
    xs = list(xs)
    if outs is None:
        outs = []
        for x in xs:
            rows, cols = x.shape
            nb = cols // block if block > 0 else 0
            outs.append((torch.empty((rows, cols // 2), dtype=torch.uint8, device=x.device),
                         torch.empty((rows, nb), dtype=torch.uint8, device=x.device),
                         torch.empty((rows, nb), dtype=torch.float32, device=x.device) if want_sse else None))
    if len(outs) != len(xs):
        raise ValueError("one output triple per tensor")
    arr = (_Tensor * max(len(xs), 1))()
    dt = None
    for i, (x, (c, s, e)) in enumerate(zip(xs, outs)):
        if not x.is_cuda or x.dim() != 2 or not x.is_contiguous():
            raise ValueError("every x must be a contiguous 2-D tensor on the GPU")
        if dt is None:
            dt = _dtype_code(x)
        elif dt != _dtype_code(x):
            raise TypeError("all tensors of a batch share one dtype")
        rows, cols = x.shape
        _need(c, rows * cols // 2, "codes_out", torch.uint8)
        _need(s, _nblocks(rows, cols, block), "scales_out", torch.uint8)
        if e is not None:
            _need(e, 4 * _nblocks(rows, cols, block), "sse_out", torch.float32)
        arr[i] = _Tensor(x.data_ptr(), rows, cols, c.data_ptr(), s.data_ptr(), e.data_ptr() if e is not None else None)
    _check(lib().mxq_quantize_batch(arr, len(xs), block, elem_fmt, scale_fmt, recipe,
                                    dt if dt is not None else DT_BF16, _stream_ptr(stream)))
    return outs


def quantize_hier(x: torch.Tensor, block: int, scale_fmt: int, recipe: int, absmax: torch.Tensor,
                  tensor_scale_out: torch.Tensor | None = None,
                  codes_out: torch.Tensor | None = None, scales_out: torch.Tensor | None = None,
                  sse_out: torch.Tensor | None = None, want_sse: bool = True, stream=None,
                  elem_fmt: int = ELEM_E2M1):
    """mxq_quantize_hier: T is derived on the device from `absmax` (the one-element tensor that
    tensor_absmax wrote).  Returns (codes, scales, sse, tensor_scale) -- the last a one-element
    fp32 device tensor."""
    if not x.is_cuda or x.dim() != 2 or not x.is_contiguous():
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, cols = x.shape
    dev = x.device
    if codes_out is None:
        codes_out = torch.empty((rows, cols // 2), dtype=torch.uint8, device=dev)
    if scales_out is None:
        scales_out = torch.empty((rows, cols // block if block > 0 else 0), dtype=torch.uint8, device=dev)
    if sse_out is None and want_sse:
        sse_out = torch.empty((rows, cols // block if block > 0 else 0), dtype=torch.float32, device=dev)
    if tensor_scale_out is None:
        tensor_scale_out = torch.ones(1, dtype=torch.float32, device=dev)
    _need(absmax, 4, "absmax", torch.float32)
    _need(tensor_scale_out, 4, "tensor_scale_out", torch.float32)
    _need(codes_out, rows * cols // 2, "codes_out", torch.uint8)
    _need(scales_out, _nblocks(rows, cols, block), "scales_out", torch.uint8)
    if sse_out is not None:
        _need(sse_out, 4 * _nblocks(rows, cols, block), "sse_out", torch.float32)
    _check(lib().mxq_quantize_hier(x.data_ptr(), rows, cols, block, elem_fmt, scale_fmt, recipe,
                                   absmax.data_ptr(), tensor_scale_out.data_ptr(), codes_out.data_ptr(),
                                   scales_out.data_ptr(), sse_out.data_ptr() if sse_out is not None else None,
                                   _dtype_code(x), _stream_ptr(stream)))
    return codes_out, scales_out, sse_out, tensor_scale_out


def dequantize(codes: torch.Tensor, scales: torch.Tensor, block: int, scale_fmt: int,
               tensor_scale=1.0, out_dtype: torch.dtype = torch.float32,
               out: torch.Tensor | None = None, stream=None, elem_fmt: int = ELEM_E2M1) -> torch.Tensor:
    """mxq_dequantize; with a one-element fp32 device tensor as `tensor_scale` (as returned by
    quantize_hier) mxq_dequantize_hier, which reads the scale on the device."""
    rows, half = codes.shape
    cols = half * 2
    if out is None:
        out = torch.empty((rows, cols), dtype=out_dtype, device=codes.device)
    _need(codes, rows * half, "codes", torch.uint8)
    _need(scales, _nblocks(rows, cols, block), "scales", torch.uint8)
    _need(out, rows * cols * out.element_size(), "out")
    if isinstance(tensor_scale, torch.Tensor):
        _need(tensor_scale, 4, "tensor_scale", torch.float32)
        _check(lib().mxq_dequantize_hier(codes.data_ptr(), scales.data_ptr(), rows, cols, block, elem_fmt,
                                         scale_fmt, tensor_scale.data_ptr(), out.data_ptr(), _dtype_code(out),
                                         _stream_ptr(stream)))
        return out
    _check(lib().mxq_dequantize(codes.data_ptr(), scales.data_ptr(), rows, cols, block, elem_fmt,
                                scale_fmt, float(tensor_scale), out.data_ptr(), _dtype_code(out),
                                _stream_ptr(stream)))
    return out


def absmax_workspace(device="cuda") -> torch.Tensor:
    """A zeroed workspace for tensor_absmax(..., workspace=...); reusable from call to call."""
    return torch.zeros(int(lib().mxq_tensor_absmax_workspace_size()), dtype=torch.uint8, device=device)


def tensor_absmax_acc(x: torch.Tensor, inout: torch.Tensor, clear_word: torch.Tensor | None = None,
                      stream=None) -> torch.Tensor:
    """mxq_tensor_absmax_acc: inout = max(inout, max |x|) in one launch; `clear_word` (optional
    one-element fp32 tensor) is zeroed for a later call."""
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor on the GPU")
    _need(inout, 4, "inout", torch.float32)
    if clear_word is not None:
        _need(clear_word, 4, "clear_word", torch.float32)
    rows = x.shape[0] if x.dim() == 2 else 1
    cols = x.shape[1] if x.dim() == 2 else x.numel()
    _check(lib().mxq_tensor_absmax_acc(x.data_ptr(), rows, cols, _dtype_code(x), inout.data_ptr(),
                                       clear_word.data_ptr() if clear_word is not None else None,
                                       _stream_ptr(stream)))
    return inout


def tensor_absmax(x: torch.Tensor, out: torch.Tensor | None = None, stream=None,
                  workspace: torch.Tensor | None = None) -> torch.Tensor:
    """mxq_tensor_absmax: one-element fp32 device tensor holding max |x|.  With a `workspace`
    (from absmax_workspace) mxq_tensor_absmax_ws, the one-launch form."""
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor on the GPU")
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=x.device)
    _need(out, 4, "out", torch.float32)
    rows = x.shape[0] if x.dim() == 2 else 1
    cols = x.shape[1] if x.dim() == 2 else x.numel()
    if workspace is not None:
        _need(workspace, 0, "workspace", torch.uint8)
        _check(lib().mxq_tensor_absmax_ws(x.data_ptr(), rows, cols, _dtype_code(x), out.data_ptr(),
                                          workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
        return out
    _check(lib().mxq_tensor_absmax(x.data_ptr(), rows, cols, _dtype_code(x), out.data_ptr(),
                                   _stream_ptr(stream)))
    return out


def tensor_absmax_static(x: torch.Tensor, out: torch.Tensor, stream=None) -> torch.Tensor:
    """mxq_tensor_absmax_static: one launch on the library's own workspace; allocates nothing
    (the output tensor is the caller's).  Calls that overlap on one GPU race."""
    if not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous tensor on the GPU")
    _need(out, 4, "out", torch.float32)
    rows = x.shape[0] if x.dim() == 2 else 1
    cols = x.shape[1] if x.dim() == 2 else x.numel()
    _check(lib().mxq_tensor_absmax_static(x.data_ptr(), rows, cols, _dtype_code(x), out.data_ptr(),
                                          _stream_ptr(stream)))
    return out


def clip_sse(x: torch.Tensor, scales: torch.Tensor, block: int, scale_fmt: int,
             tensor_scale: float = 1.0, out: torch.Tensor | None = None, stream=None,
             elem_fmt: int = ELEM_E2M1) -> torch.Tensor:
    """mxq_clip_sse: clipping-only part of the block SSE for the given scale bytes."""
    if not x.is_cuda or x.dim() != 2 or not x.is_contiguous():
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, cols = x.shape
    if out is None:
        out = torch.empty((rows, cols // block), dtype=torch.float32, device=x.device)
    _need(scales, _nblocks(rows, cols, block), "scales", torch.uint8)
    _need(out, 4 * _nblocks(rows, cols, block), "out", torch.float32)
    _check(lib().mxq_clip_sse(x.data_ptr(), scales.data_ptr(), rows, cols, block, elem_fmt, scale_fmt,
                              float(tensor_scale), out.data_ptr(), _dtype_code(x), _stream_ptr(stream)))
    return out


def histogram(codes: torch.Tensor, scales: torch.Tensor, block: int, stream=None,
              elem_fmt: int = ELEM_E2M1, out=None):
    """mxq_histogram: (int64 [8] magnitude-index counts, int64 [256] scale-byte counts); `out` may
    hold the two result tensors."""
    rows, half = codes.shape
    _need(codes, rows * half, "codes", torch.uint8)
    _need(scales, _nblocks(rows, half * 2, block), "scales", torch.uint8)
    if out is not None:
        eh, sh = out
        _need(eh, 64, "out[0]", torch.int64)
        _need(sh, 2048, "out[1]", torch.int64)
    else:
        eh = torch.empty(8, dtype=torch.int64, device=codes.device)
        sh = torch.empty(256, dtype=torch.int64, device=codes.device)
    _check(lib().mxq_histogram(codes.data_ptr(), scales.data_ptr(), rows, half * 2, block, elem_fmt,
                               eh.data_ptr(), sh.data_ptr(), _stream_ptr(stream)))
    return eh, sh


def tensor_scale_from_absmax(absmax: float, scale_fmt: int, elem_fmt: int = ELEM_E2M1) -> float:
    return float(lib().mxq_tensor_scale_from_absmax(float(absmax), elem_fmt, scale_fmt))


def scale_decode(scale_fmt: int, code: int) -> float:
    return float(lib().mxq_scale_decode(scale_fmt, int(code) & 0xFF))


def num_candidates(scale_fmt: int) -> int:
    return int(lib().mxq_num_candidates(scale_fmt))


def from_bits(bits, device="cuda") -> torch.Tensor:
    """numpy uint16 bf16 bit patterns / float32 array -> GPU tensor holding the same bytes."""
    import numpy as np
    a = np.ascontiguousarray(bits)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    if a.dtype == np.float32:
        return torch.from_numpy(a).to(device)
    raise TypeError("expected uint16 (bf16 bits) or float32")
