"""Error metrics used to gate the GPU result against the oracle.  TEST INFRASTRUCTURE ONLY.

Primary gate: max over elements of |g - r| / max(|r|, f_row) with f_row the mean |r| of the
element's row.  The floor makes the relative error meaningful where normalised outputs cross
zero; it is the continuous form of the paper's switch to absolute error below a small
constant (Section 3.2.3, the element error of the Verifier).

Secondary gate: the paper's own pass rule (same section): element error is relative above the
constant and absolute below it, and the fraction of elements whose error exceeds tau must not
exceed tau (tau = 1e-3 for fp32 in Section 4.1; no bf16 value is given there)."""
import numpy as np


def row_floor(ref: np.ndarray) -> np.ndarray:
    f = np.mean(np.abs(ref), axis=-1, keepdims=True)
    return np.where(f > 0, f, 1.0)


def max_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = np.maximum(np.abs(ref), row_floor(ref))
    e = np.abs(got - ref) / den
    return float("nan") if np.isnan(e).any() else float(np.max(e))     # (callers gate with err <= tol: NaN fails)


def max_rel_err_vec(got: np.ndarray, ref: np.ndarray) -> float:
    """Pure relative error for a vector whose entries stay away from zero (row logsumexp)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref) / np.abs(ref)))


def verifier_fraction(got: np.ndarray, ref: np.ndarray, tau: float) -> float:
    """Fraction of elements whose error (relative above the row floor, absolute below it)
    exceeds tau; the paper's rule passes when this fraction is <= tau."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    eps = np.broadcast_to(row_floor(ref), ref.shape)
    big = np.abs(ref) > eps
    e = np.where(big, np.abs(got - ref) / np.where(big, np.abs(ref), 1.0), np.abs(got - ref))
    return float(np.mean(~(e <= tau)))          # a NaN error counts as a failure
