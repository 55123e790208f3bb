"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np

TOL_F32 = 1e-5  # max |R_gpu - R_ref| / sum_k |term|, the stated fp32 tolerance
ULP_F32 = 2.0 ** -23


def worst_ratio(R_gpu: np.ndarray, R_ref: np.ndarray, abs_sum: np.ndarray, R_in=None, ulp=ULP_F32):
    """max over outputs of |R_gpu - R_ref| / sum_k |term|, the stated metric.  When the call
    accumulated into a non-zero R_in, the stored result fl(R_in + sum) carries one more rounding
    than the sum itself: an output's error is first reduced by ulp * |R_ref| (one ulp of the
    stored value: 2^-23 in fp32, 2^-52 in fp64) and what is left is held against sum_k |term|.  Outputs whose sum_k |term| is
    zero must match exactly (returns inf if one does not)."""
    denom = abs_sum.astype(np.float64)
    diff = np.abs(R_gpu.astype(np.float64) - R_ref.astype(np.float64))
    if R_in is not None and np.any(np.asarray(R_in) != 0):
        diff = np.maximum(diff - ulp * np.abs(R_ref.astype(np.float64)), 0.0)
    zero = denom == 0.0
    if np.any(diff[zero] != 0.0):
        return float("inf")
    if np.all(zero):
        return 0.0
    return float(np.max(diff[~zero] / denom[~zero]))


def assert_parity_f32(R_gpu, R_ref, abs_sum, R_in=None, tol=TOL_F32, what=""):
    assert np.all(np.isfinite(R_gpu) == np.isfinite(R_ref)), what + ": finiteness differs"
    fin = np.isfinite(R_ref)
    if not np.all(fin):
        assert np.array_equal(R_gpu[~fin], R_ref[~fin]), what + ": non-finite outputs differ"
    w = worst_ratio(np.where(fin, R_gpu, 0), np.where(fin, R_ref, 0), np.where(fin, abs_sum, 0),
                    None if R_in is None else np.where(fin, R_in, 0))
    assert w <= tol, "%s: worst |diff|/sum|term| = %.3e > %.1e" % (what, w, tol)
    return w
