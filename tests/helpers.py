"""Shared test helpers: the parity metric and its tolerances."""
import numpy as np

# Tolerances of the parity bar: max|Y - Yref| / max|Yref|.
TOL_BF16 = 2e-2   # bf16 inputs/outputs, fp32 accumulation
TOL_FP32 = 1e-5   # fp32 test mode
# IEEE half inputs/outputs, fp32 accumulation: the output rounding alone is 2^-11 = 4.9e-4 of
# |y|, the rounding of A_2 to half ahead of the down projection adds about as much at most
# (independent 2^-11 relative errors on the terms of each sum); twice their sum.
TOL_FP16 = 2e-3


def rel_err(Y, Yref) -> float:
    """Globally normalised max error: max|Y - Yref| / max|Yref|."""
    Y = np.asarray(Y, dtype=np.float64)
    Yref = np.asarray(Yref, dtype=np.float64)
    assert Y.shape == Yref.shape, (Y.shape, Yref.shape)
    if not np.all(np.isfinite(Y)):
        return float("inf")
    den = float(np.max(np.abs(Yref)))
    num = float(np.max(np.abs(Y - Yref)))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


# A second, tighter bar for the 16-bit types: the root-mean-square error over all outputs relative
# to the root-mean-square of the reference.  The maximum-norm bar above is the stated one, but for
# bf16 it is wide enough to hide a mistake that is small everywhere (one d_ff row of a few thousand
# left out of a sum changes every output by about rms(Y)/sqrt(d_ff)).  What the arithmetic predicts:
# rounding a value to p bits of precision leaves an error of rms ulp/sqrt(12), ulp = 2^(1-p) of the
# value's power of two, which over the spread of mantissas is about 2^(1-p)/sqrt(12)/1.4 of rms(Y):
# 1.6e-3 for bf16 (p = 8), 2.0e-4 for half (p = 11).  The output rounding and the rounding of A_2 ahead
# of the down projection (independent errors on the terms of each sum) contribute this much each, so
# sqrt(2) of it in all: 2.3e-3 / 2.9e-4, which is what the kernels show (2.2e-3..2.4e-3 / 2.7e-4..3.0e-4
# on every shape and candidate).  The bar is 1.5 times the prediction.  It is applied where there are
# at least 256 outputs to average over.
RMS_BF16 = 3.5e-3
RMS_FP16 = 4.4e-4
RMS_MIN_OUTPUTS = 256


def rms_err(Y, Yref) -> float:
    """rms(Y - Yref) / rms(Yref) over all elements."""
    Y = np.asarray(Y, dtype=np.float64)
    Yref = np.asarray(Yref, dtype=np.float64)
    assert Y.shape == Yref.shape, (Y.shape, Yref.shape)
    if not np.all(np.isfinite(Y)):
        return float("inf")
    den = float(np.sqrt(np.mean(Yref * Yref)))
    num = float(np.sqrt(np.mean((Y - Yref) ** 2)))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def assert_parity(Y, Yref, dtype: str, what=None) -> float:
    """The parity bar for one result: the stated maximum-norm tolerance of the type and, for the
    16-bit types, the root-mean-square bar above.  Returns the maximum-norm error."""
    tol = {"bf16": TOL_BF16, "fp16": TOL_FP16, "fp32": TOL_FP32}[dtype]
    err = rel_err(Y, Yref)
    assert err <= tol, (what, "max-norm", err, tol)
    if dtype != "fp32" and np.asarray(Yref).size >= RMS_MIN_OUTPUTS:
        bar = RMS_BF16 if dtype == "bf16" else RMS_FP16
        rms = rms_err(Y, Yref)
        assert rms <= bar, (what, "rms", rms, bar)
    return err
