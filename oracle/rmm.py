"""Algorithm 1 (forward / backward of the RMM linear layer) in fp64.

Test infrastructure.  Every function takes float64 numpy arrays (callers convert
bf16 / fp32 device tensors exactly) and performs no intermediate rounding.  S is
materialised explicitly from the state: this is the slow, obvious statement of
the algorithm, not the way the HIP path works.

Layouts follow Section 2.1: X is N x d_in (rows = tokens), W is d_out x d_in,
dY is N x d_out, X_proj is k x d_in.
"""
import numpy as np

from .sketch import sketch_S


def forward(X, W, bias, k, kind, seed, offset):
    """Algorithm 1, Forward: Y = X W^T (+ 1 b^T) (Eq. 1) and X_proj = S^T X
    (Eq. 4, second line).  Returns (Y, X_proj); the caller keeps X_proj and
    (seed, offset) in place of X."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Y = X @ W.T
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)[None, :]
    S = sketch_S(X.shape[0], k, kind, seed, offset)
    X_proj = S.T @ X
    return Y, X_proj


def backward(dY, W, X_proj, kind, seed, offset):
    """Algorithm 1, Backward: dX = dY W (Eq. 2; the listing's transposed W is a
    misprint since W is d_out x d_in), S re-made from the same state,
    dW = (dY^T S) X_proj, db = dY^T 1 (Eq. 3).  Returns (dX, dW, db)."""
    dY = np.asarray(dY, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    X_proj = np.asarray(X_proj, dtype=np.float64)
    k = X_proj.shape[0]
    dX = dY @ W
    S = sketch_S(dY.shape[0], k, kind, seed, offset)
    dW = (dY.T @ S) @ X_proj
    db = dY.sum(axis=0)
    return dX, dW, db


def sketch_apply(A, k, kind, seed, offset):
    """A (N x d) -> S^T A (k x d), the randomized-matmul primitive of Eq. 4."""
    A = np.asarray(A, dtype=np.float64)
    return sketch_S(A.shape[0], k, kind, seed, offset).T @ A


def exact_grads(X, dY):
    """Eq. 3: the gradients the estimator targets, dW = dY^T X and db = dY^T 1."""
    X = np.asarray(X, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    return dY.T @ X, dY.sum(axis=0)


def saved_bytes(n, d_in, k, elem_bytes):
    """Section 2.4.1: bytes kept for the backward pass, (RMM, plain layer).
    RMM keeps X_proj (k x d_in) and the 16-byte state; the plain layer keeps X."""
    return k * d_in * elem_bytes + 16, n * d_in * elem_bytes


def flops(n, d_in, d_out, k):
    """Section 2.4.2 with constants: multiply-add counted as 2.  Returns a dict
    of the five products of Algorithm 1 and the exact layer's three."""
    return {
        "Y": 2 * n * d_in * d_out,
        "X_proj": 2 * n * k * d_in,
        "dX": 2 * n * d_in * d_out,
        "G": 2 * n * k * d_out,
        "dW": 2 * k * d_in * d_out,
        "exact_layer": 3 * 2 * n * d_in * d_out,
    }
