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
