"""ctypes/numpy front end of the FGMP CPU oracle -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It loads oracle/libfgmp_oracle.so (built from fgmp_oracle.c by
``build()``) and never touches the HIP library.  All arithmetic is in the C
file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fgmp_oracle.c")
_LIB = os.path.join(_HERE, "libfgmp_oracle.so")
_lib = None

BLOCK = 16


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    f32p = ctypes.POINTER(ctypes.c_float)
    f64p = ctypes.POINTER(ctypes.c_double)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    i64p = ctypes.POINTER(ctypes.c_int64)
    i64 = ctypes.c_int64
    lib.fgmp_oracle_e2m1_decode.restype = ctypes.c_float
    lib.fgmp_oracle_e2m1_decode.argtypes = [ctypes.c_uint8]
    lib.fgmp_oracle_e4m3_decode.restype = ctypes.c_float
    lib.fgmp_oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
    lib.fgmp_oracle_e2m1_encode.restype = ctypes.c_uint8
    lib.fgmp_oracle_e2m1_encode.argtypes = [ctypes.c_float]
    lib.fgmp_oracle_e4m3_encode.restype = ctypes.c_uint8
    lib.fgmp_oracle_e4m3_encode.argtypes = [ctypes.c_float]
    lib.fgmp_oracle_e2m1_encode_many.restype = None
    lib.fgmp_oracle_e2m1_encode_many.argtypes = [f32p, i64, u8p]
    lib.fgmp_oracle_e4m3_encode_many.restype = None
    lib.fgmp_oracle_e4m3_encode_many.argtypes = [f32p, i64, u8p]
    lib.fgmp_oracle_quantize.restype = ctypes.c_int
    lib.fgmp_oracle_quantize.argtypes = [f32p, i64, i64, i64, f32p, i64, ctypes.c_float,
                                         ctypes.c_float, u8p, u8p, u8p, f32p]
    lib.fgmp_oracle_quantize_mode.restype = ctypes.c_int
    lib.fgmp_oracle_quantize_mode.argtypes = [f32p, i64, i64, i64, f32p, i64, ctypes.c_float,
                                              ctypes.c_float, ctypes.c_int, u8p, u8p, u8p, f32p]
    lib.fgmp_oracle_quantize_clip.restype = ctypes.c_int
    lib.fgmp_oracle_quantize_clip.argtypes = [f32p, i64, i64, i64, f32p, i64, ctypes.c_float,
                                              ctypes.c_float, u8p, u8p, u8p, f32p]
    lib.fgmp_oracle_dequantize.restype = ctypes.c_int
    lib.fgmp_oracle_dequantize.argtypes = [u8p, u8p, u8p, i64, i64, f64p]
    lib.fgmp_oracle_gemm.restype = ctypes.c_int
    lib.fgmp_oracle_gemm.argtypes = [f64p, ctypes.c_double, f64p, ctypes.c_double, i64,
                                     i64p, i64, i64p, i64, f64p, f64p]
    lib.fgmp_oracle_exp_steps.restype = ctypes.c_float
    lib.fgmp_oracle_exp_steps.argtypes = [ctypes.c_float]
    lib.fgmp_oracle_silu_mul.restype = None
    lib.fgmp_oracle_silu_mul.argtypes = [f32p, f32p, i64, f32p]
    lib.fgmp_oracle_exp_rounded_once.restype = ctypes.c_float
    lib.fgmp_oracle_exp_rounded_once.argtypes = [ctypes.c_float]
    lib.fgmp_oracle_silu_mul_rounded_once.restype = None
    lib.fgmp_oracle_silu_mul_rounded_once.argtypes = [f32p, f32p, i64, f32p]
    lib.fgmp_oracle_threshold.restype = ctypes.c_float
    lib.fgmp_oracle_threshold.argtypes = [f32p, i64, ctypes.c_double]
    lib.fgmp_oracle_storage_bits.restype = i64
    lib.fgmp_oracle_storage_bits.argtypes = [i64, i64]
    lib.fgmp_oracle_num_threads.restype = ctypes.c_int
    lib.fgmp_oracle_num_threads.argtypes = []
    lib.fgmp_oracle_set_num_threads.restype = None
    lib.fgmp_oracle_set_num_threads.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def e2m1_decode(code: int) -> float:
    return float(_load().fgmp_oracle_e2m1_decode(int(code) & 0xFF))


def e4m3_decode(code: int) -> float:
    return float(_load().fgmp_oracle_e4m3_decode(int(code) & 0xFF))


def e2m1_encode(r) -> np.ndarray:
    """Elementwise fp32 -> E2M1 code (0..15)."""
    a = np.ascontiguousarray(np.asarray(r, dtype=np.float32)).reshape(-1)
    out = np.empty(a.size, dtype=np.uint8)
    _load().fgmp_oracle_e2m1_encode_many(_ptr(a, ctypes.c_float), a.size, _ptr(out, ctypes.c_uint8))
    return out.reshape(np.shape(r))


def e4m3_encode(r) -> np.ndarray:
    """Elementwise fp32 -> E4M3 code byte."""
    a = np.ascontiguousarray(np.asarray(r, dtype=np.float32)).reshape(-1)
    out = np.empty(a.size, dtype=np.uint8)
    _load().fgmp_oracle_e4m3_encode_many(_ptr(a, ctypes.c_float), a.size, _ptr(out, ctypes.c_uint8))
    return out.reshape(np.shape(r))


SCORE_MODES = {"nvfp4_error": 0, "delta": 1}


def quantize(x: np.ndarray, fisher: np.ndarray, threshold: float, scale: float, score_mode: str = "nvfp4_error",
             clip: bool = False):
    """Quantize a rows x K fp32 tensor.  fisher is (K,) per channel or (rows, K)
    per element.  score_mode: "nvfp4_error" (Eq. 6) or "delta" (Eq. 8).
    clip: choose each block scale by sensitivity-weighted clipping (Eq. 11).
    Returns dict(codes, scales, mask, scores)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    fisher = np.ascontiguousarray(fisher, dtype=np.float32)
    rows, K = x.shape
    if fisher.ndim == 1:
        assert fisher.shape == (K,)
        ldf = 0
    else:
        assert fisher.shape == (rows, K)
        ldf = K
    nb = K // BLOCK
    codes = np.empty((rows, K), dtype=np.uint8)
    scales = np.empty((rows, nb), dtype=np.uint8)
    mask = np.empty((rows, nb), dtype=np.uint8)
    scores = np.empty((rows, nb), dtype=np.float32)
    if clip:
        if score_mode != "nvfp4_error":
            raise ValueError("clipping is defined with the NVFP4-error score")
        rc = _load().fgmp_oracle_quantize_clip(_ptr(x, ctypes.c_float), rows, K, K,
                                               _ptr(fisher, ctypes.c_float), ldf,
                                               ctypes.c_float(threshold), ctypes.c_float(scale),
                                               _ptr(codes, ctypes.c_uint8), _ptr(scales, ctypes.c_uint8),
                                               _ptr(mask, ctypes.c_uint8), _ptr(scores, ctypes.c_float))
        if rc != 0:
            raise ValueError("fgmp_oracle_quantize_clip: bad argument or non-finite input")
        return {"codes": codes, "scales": scales, "mask": mask, "scores": scores}
    rc = _load().fgmp_oracle_quantize_mode(_ptr(x, ctypes.c_float), rows, K, K,
                                           _ptr(fisher, ctypes.c_float), ldf,
                                           ctypes.c_float(threshold), ctypes.c_float(scale),
                                           SCORE_MODES[score_mode],
                                           _ptr(codes, ctypes.c_uint8), _ptr(scales, ctypes.c_uint8),
                                           _ptr(mask, ctypes.c_uint8), _ptr(scores, ctypes.c_float))
    if rc != 0:
        raise ValueError("fgmp_oracle_quantize: bad argument or non-finite input")
    return {"codes": codes, "scales": scales, "mask": mask, "scores": scores}


def dequantize(codes: np.ndarray, scales: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Real value of each stored element, without the tensor scale (fp64)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    rows, K = codes.shape
    out = np.empty((rows, K), dtype=np.float64)
    rc = _load().fgmp_oracle_dequantize(_ptr(codes, ctypes.c_uint8), _ptr(scales, ctypes.c_uint8),
                                        _ptr(mask, ctypes.c_uint8), rows, K,
                                        _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("fgmp_oracle_dequantize: bad argument")
    return out


def gemm(ax: np.ndarray, sx: float, aw: np.ndarray, sw: float, rows=None, cols=None):
    """Y = sx*sw * ax @ aw.T restricted to the given rows of ax / rows of aw,
    with the per-element tolerance 1e-5 * sx*sw * sum_k |ax*aw|."""
    ax = np.ascontiguousarray(ax, dtype=np.float64)
    aw = np.ascontiguousarray(aw, dtype=np.float64)
    K = ax.shape[1]
    assert aw.shape[1] == K
    ri = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    ci = None if cols is None else np.ascontiguousarray(cols, dtype=np.int64)
    nr = ax.shape[0] if ri is None else ri.size
    nc = aw.shape[0] if ci is None else ci.size
    Y = np.empty((nr, nc), dtype=np.float64)
    tol = np.empty((nr, nc), dtype=np.float64)
    rc = _load().fgmp_oracle_gemm(_ptr(ax, ctypes.c_double), float(sx), _ptr(aw, ctypes.c_double),
                                  float(sw), K,
                                  None if ri is None else _ptr(ri, ctypes.c_int64), nr,
                                  None if ci is None else _ptr(ci, ctypes.c_int64), nc,
                                  _ptr(Y, ctypes.c_double), _ptr(tol, ctypes.c_double))
    if rc != 0:
        raise ValueError("fgmp_oracle_gemm: bad argument")
    return Y, tol


def exp_steps(x: float) -> float:
    """The fp32 exponential the gated activation is defined with (see the C source)."""
    return float(_load().fgmp_oracle_exp_steps(float(np.float32(x))))


def silu_mul(g: np.ndarray, u: np.ndarray) -> np.ndarray:
    """h = SiLU(g) * u, elementwise, in the fixed fp32 sequence of the C source."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    if g.shape != u.shape:
        raise ValueError("silu_mul: shapes differ")
    h = np.empty_like(g)
    _load().fgmp_oracle_silu_mul(_ptr(g, ctypes.c_float), _ptr(u, ctypes.c_float), g.size, _ptr(h, ctypes.c_float))
    return h


def exp_rounded_once(x: float) -> float:
    """e^x (x clamped to [-87, 88]) from the fp64 library exponential, rounded to fp32 once: the
    cross-check of exp_steps, written without range reduction or polynomial."""
    return float(_load().fgmp_oracle_exp_rounded_once(float(np.float32(x))))


def silu_mul_rounded_once(g: np.ndarray, u: np.ndarray) -> np.ndarray:
    """The fp32 nearest to g / (1 + e^-g) * u evaluated in fp64: the cross-check of silu_mul."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    if g.shape != u.shape:
        raise ValueError("silu_mul_rounded_once: shapes differ")
    h = np.empty_like(g)
    _load().fgmp_oracle_silu_mul_rounded_once(_ptr(g, ctypes.c_float), _ptr(u, ctypes.c_float), g.size,
                                              _ptr(h, ctypes.c_float))
    return h


def gate_columns(y: np.ndarray) -> np.ndarray:
    """The gated activation over a product whose columns come in groups of 64: columns 64q .. 64q+31 are
    the gate values of hidden units 32q .. 32q+31, columns 64q+32 .. 64q+63 their up values."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    if y.ndim != 2 or y.shape[1] % 64 != 0:
        raise ValueError("gate_columns: the column count must be a multiple of 64")
    v = y.reshape(y.shape[0], y.shape[1] // 64, 2, 32)
    return silu_mul(v[:, :, 0, :], v[:, :, 1, :]).reshape(y.shape[0], y.shape[1] // 2)


def threshold(scores: np.ndarray, fraction: float) -> float:
    s = np.ascontiguousarray(scores, dtype=np.float32).reshape(-1)
    return float(_load().fgmp_oracle_threshold(_ptr(s, ctypes.c_float), s.size, float(fraction)))


def storage_bits(n_lo: int, n_hi: int) -> int:
    return int(_load().fgmp_oracle_storage_bits(int(n_lo), int(n_hi)))


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    return int(_load().fgmp_oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the OpenMP loops of the oracle use from now on."""
    _load().fgmp_oracle_set_num_threads(int(n))
