"""Closed-form variances around the RMM estimate (Section 2.3), fp64.

Test infrastructure.  X is N x d_in, Y (= dY) is N x d_out; the estimate is
dW_rmm = Y^T S S^T X with S as in oracle.sketch.

Reading of Lemma 2.2: as printed, D^2_RMM = (|X|^2 |Y|^2 - |X^T Y|^2) / k.  The
proof's equal-index case treats E[C^2 C^2] as E[C^2] E[C^2] also when both
factors are the same Gaussian entry, which drops the fourth moment (3, not 1).
Carrying it gives a plus sign; `rmm_variance_gaussian` is that corrected form
and `d2_rmm_printed` the lemma as printed (the two agree when X^T Y = 0, which
is the case in the paper's worked example).
"""
import numpy as np


def _f64(*arrs):
    return tuple(np.asarray(a, dtype=np.float64) for a in arrs)


def inner_product_variance(a, b, k, kind_rademacher=False):
    """Var[a^T S S^T b] for vectors a, b of length N:
    (|a|^2 |b|^2 + (a.b)^2) / k for Gaussian S, and 2 sum_i a_i^2 b_i^2 / k less
    for Rademacher S."""
    a, b = _f64(a, b)
    v = (a @ a) * (b @ b) + (a @ b) ** 2
    if kind_rademacher:
        v -= 2.0 * np.sum(a * a * b * b)
    return v / k


def rmm_variance_gaussian(X, Y, k):
    """E |Y^T S S^T X - Y^T X|_F^2 for Gaussian S (Lemma 2.2, corrected sign)."""
    X, Y = _f64(X, Y)
    return (np.sum(X * X) * np.sum(Y * Y) + np.sum((Y.T @ X) ** 2)) / k


def rmm_variance_rademacher(X, Y, k):
    """Same expectation for Rademacher S: the Gaussian value minus
    2 sum_i |x_i|^2 |y_i|^2 / k (x_i, y_i the i-th rows)."""
    X, Y = _f64(X, Y)
    rows = np.sum(np.sum(X * X, axis=1) * np.sum(Y * Y, axis=1))
    return rmm_variance_gaussian(X, Y, k) - 2.0 * rows / k


def d2_rmm_printed(X, Y, k):
    """Lemma 2.2 exactly as printed (minus sign); kept for the worked example."""
    X, Y = _f64(X, Y)
    return (np.sum(X * X) * np.sum(Y * Y) - np.sum((X.T @ Y) ** 2)) / k


def d2_sgd(X, Y):
    """Lemma 2.1: B/(B-1) sum_k |x_k|^2 |y_k|^2 - |X^T Y|_F^2 / (B-1)."""
    X, Y = _f64(X, Y)
    B = X.shape[0]
    rows = np.sum(np.sum(X * X, axis=1) * np.sum(Y * Y, axis=1))
    return B / (B - 1.0) * rows - np.sum((X.T @ Y) ** 2) / (B - 1.0)


def alpha(X, Y):
    """Theorem 2.3: alpha = |X^T Y|_F^2 / (|X|_F^2 |Y|_F^2), in [0, 1]."""
    X, Y = _f64(X, Y)
    return np.sum((X.T @ Y) ** 2) / (np.sum(X * X) * np.sum(Y * Y))
