"""CPU oracle package.  TEST INFRASTRUCTURE ONLY.

Holds the plain, slow, double-precision statement of what the GPU path computes:

* ``conv2d_fwd`` / ``conv2d_fwd_point`` -- forward convolution by its definition
  (C code in ``conv_oracle.c``; the paper's Fig. 4 with the channel blocking undone);
* ``layout`` -- the blocked tensor layouts of Fig. 4 written as index identities in numpy;
* ``reuse_oracle`` -- Section 4's working-set analysis and cost function by brute-force enumeration;
* ``ranker_oracle`` -- Section 4.2.2's pairwise network and tournament in float64 numpy.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It imports nothing from the GPU package and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_conv.so")
_lock = threading.Lock()
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP).  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"],
            check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            dp = ctypes.POINTER(ctypes.c_double)
            fp = ctypes.POINTER(ctypes.c_float)
            ip = ctypes.POINTER(ctypes.c_int32)
            sp = ctypes.POINTER(_Shape)
            lib.oracle_out_dims.argtypes = [sp, ip, ip]
            lib.oracle_conv2d_fwd.argtypes = [sp, fp, fp, dp, dp]
            lib.oracle_conv2d_fwd_range.argtypes = [sp, fp, fp, dp, dp, ctypes.c_int32, ctypes.c_int32]
            lib.oracle_conv2d_fwd_point.argtypes = [sp, fp, fp] + [ctypes.c_int32] * 4 + [dp, dp]
            lib.oracle_threads.restype = ctypes.c_int
            _lib = lib
    return _lib


def _shape_struct(shape) -> _Shape:
    return _Shape(*(int(getattr(shape, f)) for f in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")))


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().oracle_threads())


def out_dims(shape) -> tuple[int, int]:
    P, Q = ctypes.c_int32(), ctypes.c_int32()
    if _load().oracle_out_dims(ctypes.byref(_shape_struct(shape)), ctypes.byref(P), ctypes.byref(Q)) != 0:
        raise ValueError(f"invalid convolution shape {shape}")
    return P.value, Q.value


def _check_inputs(shape, x, w):
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    if x.shape != (shape.N, shape.C, shape.H, shape.W):
        raise ValueError(f"input shape {x.shape} does not match {shape}")
    if w.shape != (shape.K, shape.C, shape.R, shape.S):
        raise ValueError(f"filter shape {w.shape} does not match {shape}")
    return x, w


def conv2d_fwd(shape, x: np.ndarray, w: np.ndarray, images: tuple[int, int] | None = None):
    """Forward convolution by definition, fp64 accumulate.

    x: NCHW fp32, w: KCRS fp32.  Returns (out, mag), both NKPQ fp64; ``mag`` is the sum of
    |x*w| over the same terms.  ``images=(n0, n1)`` computes only that image range (the rest
    of the returned arrays is zero)."""
    x, w = _check_inputs(shape, x, w)
    P, Q = out_dims(shape)
    out = np.zeros((shape.N, shape.K, P, Q), dtype=np.float64)
    mag = np.zeros_like(out)
    n0, n1 = (0, shape.N) if images is None else images
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().oracle_conv2d_fwd_range(
        ctypes.byref(_shape_struct(shape)), x.ctypes.data_as(fp), w.ctypes.data_as(fp),
        out.ctypes.data_as(dp), mag.ctypes.data_as(dp), int(n0), int(n1))
    if rc != 0:
        raise ValueError(f"oracle rejected shape {shape} / image range {images}")
    return out, mag


def conv2d_fwd_point(shape, x: np.ndarray, w: np.ndarray, n: int, k: int, p: int, q: int):
    """One output element (value, magnitude) -- for sampled checks of large layers."""
    x, w = _check_inputs(shape, x, w)
    o, m = ctypes.c_double(), ctypes.c_double()
    fp = ctypes.POINTER(ctypes.c_float)
    rc = _load().oracle_conv2d_fwd_point(
        ctypes.byref(_shape_struct(shape)), x.ctypes.data_as(fp), w.ctypes.data_as(fp),
        int(n), int(k), int(p), int(q), ctypes.byref(o), ctypes.byref(m))
    if rc != 0:
        raise ValueError("oracle rejected point query")
    return o.value, m.value


def normalised_error(got: np.ndarray, out: np.ndarray, mag: np.ndarray) -> float:
    """max |got - out| / mag over all outputs; an output whose magnitude is exactly zero
    must itself be exactly zero (else the error is infinite)."""
    got = np.asarray(got, dtype=np.float64)
    diff = np.abs(got - out)
    zero = mag == 0.0
    if np.any(diff[zero] != 0.0):
        return float("inf")
    if np.all(zero):
        return 0.0
    return float(np.max(diff[~zero] / mag[~zero]))


def round_to_bf16(y: np.ndarray) -> np.ndarray:
    """Finite float64 values rounded to the nearest bfloat16 (8 significant bits), ties to even; result as float64."""
    y = np.asarray(y, dtype=np.float64)
    m, e = np.frexp(y)                       # y = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # np.rint rounds half to even


def conv2d_fwd_fused(shape, x: np.ndarray, w: np.ndarray, bias: np.ndarray | None = None, relu: bool = False,
                     out_bf16: bool = False):
    """What follows a convolution in an inference pipeline, applied to the exact result in this order:
    per-output-channel bias, max(., 0), rounding of the output to bfloat16.  Returns (y, mag, y_before_rounding)
    with mag = sum |x*w| + |bias|, the scale the accumulation error is measured against."""
    out, mag = conv2d_fwd(shape, x, w)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64).reshape(1, -1, 1, 1)
        out = out + b
        mag = mag + np.abs(b)
    if relu:
        out = np.maximum(out, 0.0)
    exact = out
    if out_bf16:
        out = round_to_bf16(out)
    return out, mag, exact
