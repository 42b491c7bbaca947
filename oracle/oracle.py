"""ctypes front end of the fp64 CPU oracle (TEST INFRASTRUCTURE ONLY).

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module; the product path never does.  It wraps
``swiglu_oracle.c`` (built with plain gcc into ``liboracle.so`` next to this
file) and does argument marshalling only: all arithmetic is in the C file,
which follows the SwiGLU equations of the Background section and the
two-stage split of the Method section.

Arrays are numpy: bfloat16 tensors are passed as their uint16 bit patterns,
fp32 tensors as float32, IEEE half tensors as float16.  Layouts: X [M, d_model]; W_gate, W_up, W_down all
[d_ff, d_model] row-major; results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swiglu_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

BF16 = 0
FP32 = 1
FP16 = 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
             "-o", _LIB, _SRC, "-lm", "-lpthread"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, dp, ci = ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.c_int
        lib.oracle_silu.restype = ctypes.c_double
        lib.oracle_silu.argtypes = [ctypes.c_double]
        lib.oracle_gate_up_silu.restype = ci
        lib.oracle_gate_up_silu.argtypes = [vp, vp, vp, dp, dp, dp, ci, ci, ci, ci, ci]
        lib.oracle_down.restype = ci
        lib.oracle_down.argtypes = [dp, vp, dp, ci, ci, ci, ci, ci]
        lib.oracle_rmsnorm.restype = ci
        lib.oracle_rmsnorm.argtypes = [vp, vp, dp, ci, ci, ci, ctypes.c_double]
        lib.oracle_mlp_block.restype = ci
        lib.oracle_mlp_block.argtypes = [vp, vp, ctypes.c_double, vp, vp, vp, dp, ci, ci, ci, ci, ci]
        lib.oracle_swiglu_mlp.restype = ci
        lib.oracle_swiglu_mlp.argtypes = [vp, vp, vp, vp, dp, ci, ci, ci, ci, ci]
        _lib = lib
    return _lib


def default_threads() -> int:
    return max(1, len(os.sched_getaffinity(0)))


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return FP32
    if a.dtype == np.float16:
        return FP16
    raise TypeError(f"oracle takes uint16 (bf16 bits), float16 or float32 arrays, got {a.dtype}")


def _prep(a: np.ndarray, shape, code: int) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if _dtype_code(a) != code:
        raise TypeError("all oracle inputs must share one element type")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def silu(g: float) -> float:
    """SiLU(g) = Sigmoid(g) * g, in fp64 (Background, SwiGLU equations)."""
    return float(_load().oracle_silu(float(g)))


def gate_up_silu(X, Wg, Wu, nthreads: int | None = None):
    """Stage one: returns (A_gate, A_1, A_2), each float64 [M, d_ff]."""
    X = np.ascontiguousarray(X)
    code = _dtype_code(X)
    M, d_model = X.shape
    d_ff = Wg.shape[0]
    Wg = _prep(Wg, (d_ff, d_model), code)
    Wu = _prep(Wu, (d_ff, d_model), code)
    G = np.empty((M, d_ff), np.float64)
    U = np.empty((M, d_ff), np.float64)
    A2 = np.empty((M, d_ff), np.float64)
    rc = _load().oracle_gate_up_silu(
        X.ctypes.data, Wg.ctypes.data, Wu.ctypes.data, _dptr(G), _dptr(U), _dptr(A2),
        M, d_model, d_ff, code, nthreads or default_threads())
    if rc != 0:
        raise RuntimeError(f"oracle_gate_up_silu failed with {rc}")
    return G, U, A2


def down(A2, Wd, nthreads: int | None = None):
    """Stage two: Y = A_2 W_down, float64 [M, d_model]; A_2 given in float64."""
    A2 = np.ascontiguousarray(A2, dtype=np.float64)
    Wd = np.ascontiguousarray(Wd)
    code = _dtype_code(Wd)
    M, d_ff = A2.shape
    d_model = Wd.shape[1]
    Wd = _prep(Wd, (d_ff, d_model), code)
    Y = np.empty((M, d_model), np.float64)
    rc = _load().oracle_down(_dptr(A2), Wd.ctypes.data, _dptr(Y), M, d_model, d_ff, code,
                             nthreads or default_threads())
    if rc != 0:
        raise RuntimeError(f"oracle_down failed with {rc}")
    return Y


def swiglu_mlp(X, Wg, Wu, Wd, nthreads: int | None = None):
    """Y = (SiLU(X W_gate) (x) (X W_up)) W_down, float64 [M, d_model]."""
    X = np.ascontiguousarray(X)
    code = _dtype_code(X)
    M, d_model = X.shape
    d_ff = Wg.shape[0]
    Wg = _prep(Wg, (d_ff, d_model), code)
    Wu = _prep(Wu, (d_ff, d_model), code)
    Wd = _prep(Wd, (d_ff, d_model), code)
    Y = np.empty((M, d_model), np.float64)
    rc = _load().oracle_swiglu_mlp(
        X.ctypes.data, Wg.ctypes.data, Wu.ctypes.data, Wd.ctypes.data, _dptr(Y),
        M, d_model, d_ff, code, nthreads or default_threads())
    if rc != 0:
        raise RuntimeError(f"oracle_swiglu_mlp failed with {rc}")
    return Y


def rmsnorm(H, w=None, eps: float = 0.0):
    """N = H * w / sqrt(mean_k(H^2) + eps) row by row, float64 [M, d_model] (w None = ones)."""
    H = np.ascontiguousarray(H)
    code = _dtype_code(H)
    M, d_model = H.shape
    wp = None
    if w is not None:
        w = _prep(w, (d_model,), code)
        wp = w.ctypes.data
    N = np.empty((M, d_model), np.float64)
    rc = _load().oracle_rmsnorm(H.ctypes.data, wp, _dptr(N), M, d_model, code, float(eps))
    if rc != 0:
        raise RuntimeError(f"oracle_rmsnorm failed with {rc}")
    return N


def mlp_block(H, w, eps, Wg, Wu, Wd, nthreads: int | None = None):
    """H_out = H + SwiGLU_MLP(RMSNorm(H; w, eps)), float64 [M, d_model]."""
    H = np.ascontiguousarray(H)
    code = _dtype_code(H)
    M, d_model = H.shape
    d_ff = Wg.shape[0]
    Wg = _prep(Wg, (d_ff, d_model), code)
    Wu = _prep(Wu, (d_ff, d_model), code)
    Wd = _prep(Wd, (d_ff, d_model), code)
    wp = None
    if w is not None:
        w = _prep(w, (d_model,), code)
        wp = w.ctypes.data
    Y = np.empty((M, d_model), np.float64)
    rc = _load().oracle_mlp_block(H.ctypes.data, wp, float(eps), Wg.ctypes.data, Wu.ctypes.data,
                                  Wd.ctypes.data, _dptr(Y), M, d_model, d_ff, code,
                                  nthreads or default_threads())
    if rc != 0:
        raise RuntimeError(f"oracle_mlp_block failed with {rc}")
    return Y
