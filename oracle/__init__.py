"""CPU oracle for microscaled FP4 quantisation -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy wrapper over ``mxq_oracle.c`` (see that file's header for what is computed
and which passages of the paper each step follows).  Nothing in the product package imports
this module; only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg do.
The wrapper holds no arithmetic of the method: it marshals numpy arrays into the C calls.

bf16 tensors are passed as ``numpy.uint16`` arrays holding the bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mxq_oracle.c")
_LIB = os.path.join(_HERE, "libmxq_oracle.so")

DT_BF16, DT_F32 = 0, 1
SCALE_E8M0, SCALE_E4M3, SCALE_UE5M3 = 0, 1, 2
ABSMAX, ABSMAX_PZ, FOUR_OVER_SIX, FOUR_OVER_SIX_PZ, BRUTE = 0, 1, 2, 3, 4
SEL_PINNED, SEL_EXACT = 0, 1

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    i64, i32, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_float
    vp = ctypes.c_void_p
    lib.orc_e2m1_decode.restype = f32
    lib.orc_e2m1_decode.argtypes = [i32]
    lib.orc_scale_decode.restype = f32
    lib.orc_scale_decode.argtypes = [i32, i32]
    lib.orc_scale_max_code.restype = i32
    lib.orc_scale_max_code.argtypes = [i32]
    lib.orc_num_candidates.restype = i32
    lib.orc_num_candidates.argtypes = [i32]
    lib.orc_scale_eps.restype = f32
    lib.orc_scale_eps.argtypes = [i32]
    lib.orc_round_sf.restype = i32
    lib.orc_round_sf.argtypes = [i32, f32]
    lib.orc_pow2_code.restype = i32
    lib.orc_pow2_code.argtypes = [f32, f32]
    lib.orc_e2m1_round_mag.restype = i32
    lib.orc_e2m1_round_mag.argtypes = [f32]
    lib.orc_quantize.restype = i32
    lib.orc_quantize.argtypes = [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp, vp, vp, vp]
    lib.orc_block_sse.restype = i32
    lib.orc_block_sse.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    lib.orc_clip_sse.restype = i32
    lib.orc_clip_sse.argtypes = [vp, i32, i64, i64, i32, i32, f32, vp, vp]
    lib.orc_dequantize.restype = i32
    lib.orc_dequantize.argtypes = [vp, vp, i64, i64, i32, i32, f32, vp, i32]
    lib.orc_tensor_absmax.restype = f32
    lib.orc_tensor_absmax.argtypes = [vp, i32, i64]
    lib.orc_tensor_scale.restype = f32
    lib.orc_tensor_scale.argtypes = [f32, i32]
    lib.orc_num_threads.restype = i32
    lib.orc_set_num_threads.argtypes = [i32]
    _lib = lib
    return lib


def _dtype_of(x: np.ndarray) -> int:
    if x.dtype == np.uint16:
        return DT_BF16
    if x.dtype == np.float32:
        return DT_F32
    raise TypeError("oracle input must be float32 or uint16 (bf16 bit patterns)")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def e2m1_decode(code: int) -> float:
    return float(_load().orc_e2m1_decode(int(code)))


def e2m1_round_mag(y: float) -> int:
    return int(_load().orc_e2m1_round_mag(float(np.float32(y))))


def scale_decode(fmt: int, code: int) -> float:
    return float(_load().orc_scale_decode(fmt, int(code)))


def scale_max_code(fmt: int) -> int:
    return int(_load().orc_scale_max_code(fmt))


def num_candidates(fmt: int) -> int:
    return int(_load().orc_num_candidates(fmt))


def scale_eps(fmt: int) -> float:
    return float(_load().orc_scale_eps(fmt))


def round_sf(fmt: int, r: float) -> int:
    return int(_load().orc_round_sf(fmt, float(np.float32(r))))


def pow2_code(amax: float, M: float = 6.0) -> int:
    return int(_load().orc_pow2_code(float(np.float32(amax)), float(M)))


def quantize(x: np.ndarray, block: int, scale_fmt: int, recipe: int,
             tensor_scale: float = 1.0, sel_mode: int = SEL_PINNED, want_exact: bool = False):
    """Returns (codes u8 [R, C/2], scales u8 [R, C/block], sse f32 [R, C/block]) and, when
    ``want_exact``, a fourth array with the long-double SSE of the selected candidate."""
    x = np.ascontiguousarray(x)
    assert x.ndim == 2
    rows, cols = x.shape
    nbc = cols // block if block > 0 else 0
    codes = np.empty((rows, cols // 2), np.uint8)
    scales = np.empty((rows, nbc), np.uint8)
    sse = np.empty((rows, nbc), np.float32)
    ex = np.empty((rows, nbc), np.float64) if want_exact else None
    rc = _load().orc_quantize(_ptr(x), _dtype_of(x), rows, cols, block, scale_fmt, recipe,
                              float(np.float32(tensor_scale)), sel_mode, _ptr(codes),
                              _ptr(scales), _ptr(sse), _ptr(ex) if want_exact else None)
    if rc != 0:
        raise ValueError(f"orc_quantize rejected its arguments (rc={rc})")
    return (codes, scales, sse, ex) if want_exact else (codes, scales, sse)


def block_sse(v: np.ndarray, scale_fmt: int, code: int):
    """(codes4 u8 [b], pinned fp32 SSE, exact SSE) of one block under one scale code."""
    v = np.ascontiguousarray(v, np.float32)
    b = v.shape[0]
    c4 = np.empty(b, np.uint8)
    sp = np.empty(1, np.float32)
    se = np.empty(1, np.float64)
    rc = _load().orc_block_sse(_ptr(v), b, scale_fmt, int(code), _ptr(c4), _ptr(sp), _ptr(se))
    if rc != 0:
        raise ValueError("orc_block_sse rejected its arguments")
    return c4, sp[0], se[0]


def dequantize(codes: np.ndarray, scales: np.ndarray, block: int, scale_fmt: int,
               tensor_scale: float = 1.0, out_dtype: int = DT_F32) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.uint8)
    rows, half = codes.shape
    cols = half * 2
    out = np.empty((rows, cols), np.float32 if out_dtype == DT_F32 else np.uint16)
    rc = _load().orc_dequantize(_ptr(codes), _ptr(scales), rows, cols, block, scale_fmt,
                                float(np.float32(tensor_scale)), _ptr(out), out_dtype)
    if rc != 0:
        raise ValueError("orc_dequantize rejected its arguments")
    return out


def clip_sse(x: np.ndarray, scales: np.ndarray, block: int, scale_fmt: int,
             tensor_scale: float = 1.0) -> np.ndarray:
    """Clipping-only block SSE for the given scale bytes (f32 [R, C/block])."""
    x = np.ascontiguousarray(x)
    scales = np.ascontiguousarray(scales, np.uint8)
    rows, cols = x.shape
    out = np.empty((rows, cols // block), np.float32)
    rc = _load().orc_clip_sse(_ptr(x), _dtype_of(x), rows, cols, block, scale_fmt,
                              float(np.float32(tensor_scale)), _ptr(scales), _ptr(out))
    if rc != 0:
        raise ValueError("orc_clip_sse rejected its arguments")
    return out


def histograms(codes: np.ndarray, scales: np.ndarray):
    """Appendix histograms: counts of the 8 E2M1 magnitude indices over all elements and of the
    256 scale bytes over all blocks (uint64 [8], uint64 [256])."""
    codes = np.ascontiguousarray(codes, np.uint8).ravel()
    mags = np.concatenate([codes & 7, (codes >> 4) & 7])
    return (np.bincount(mags, minlength=8).astype(np.uint64),
            np.bincount(np.ascontiguousarray(scales, np.uint8).ravel(), minlength=256).astype(np.uint64))


def tensor_absmax(x: np.ndarray) -> float:
    x = np.ascontiguousarray(x)
    return float(_load().orc_tensor_absmax(_ptr(x), _dtype_of(x), x.size))


def tensor_scale(absmax: float, scale_fmt: int) -> float:
    return float(_load().orc_tensor_scale(float(np.float32(absmax)), scale_fmt))


def tensor_mse(sse: np.ndarray, n_elements: int, tensor_scale_: float = 1.0) -> float:
    """Per-tensor MSE in the original domain: T^2 * sum(block SSE) / (R*C), in float64."""
    t = float(np.float32(tensor_scale_))
    return t * t * float(np.sum(sse, dtype=np.float64)) / float(n_elements)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(int(n))
