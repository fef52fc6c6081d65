"""Pins for oracle.rmm: brute-force loops on tiny inputs (Eq. 1-3), the estimator
written two ways (Eq. 4), Monte-Carlo unbiasedness, memory and flop formulas
(Section 2.4, Table 1)."""
import math

import numpy as np

from oracle import rmm, sketch


def _tiny(seed, n=5, d_in=3, d_out=4):
    g = np.random.default_rng(seed)
    return g.standard_normal((n, d_in)), g.standard_normal((d_out, d_in)), \
        g.standard_normal(d_out), g.standard_normal((n, d_out))


def test_forward_backward_against_triple_loops():
    X, W, b, dY = _tiny(1)
    n, d_in = X.shape
    d_out = W.shape[0]
    k, kind, seed, off = 3, sketch.GAUSSIAN, 42, 9
    S = sketch.sketch_S(n, k, kind, seed, off)
    Y, Xp = rmm.forward(X, W, b, k, kind, seed, off)
    dX, dW, db = rmm.backward(dY, W, Xp, kind, seed, off)
    for i in range(n):
        for o in range(d_out):
            acc = b[o]
            for c in range(d_in):
                acc += X[i, c] * W[o, c]
            assert abs(Y[i, o] - acc) < 1e-12
    for r in range(k):
        for c in range(d_in):
            acc = 0.0
            for i in range(n):
                acc += S[i, r] * X[i, c]
            assert abs(Xp[r, c] - acc) < 1e-12
    for i in range(n):
        for c in range(d_in):
            acc = 0.0
            for o in range(d_out):
                acc += dY[i, o] * W[o, c]
            assert abs(dX[i, c] - acc) < 1e-12
    for o in range(d_out):
        acc_b = 0.0
        for i in range(n):
            acc_b += dY[i, o]
        assert abs(db[o] - acc_b) < 1e-12
        for c in range(d_in):
            acc = 0.0
            for r in range(k):
                g = 0.0
                for i in range(n):
                    g += S[i, r] * dY[i, o]
                acc += g * Xp[r, c]
            assert abs(dW[o, c] - acc) < 1e-12


def test_hand_checkable_2x2():
    X = np.array([[1.0, 2.0], [3.0, 4.0]])
    W = np.array([[1.0, 0.0], [1.0, 1.0]])        # d_out x d_in
    dY = np.array([[1.0, 0.0], [0.0, 2.0]])
    Y, _ = rmm.forward(X, W, None, 1, sketch.GAUSSIAN, 0, 0)
    assert Y.tolist() == [[1.0, 3.0], [3.0, 7.0]]
    dX, _, db = rmm.backward(dY, W, np.zeros((1, 2)), sketch.GAUSSIAN, 0, 0)
    assert dX.tolist() == [[1.0, 0.0], [2.0, 2.0]]
    assert db.tolist() == [1.0, 2.0]
    dW, db2 = rmm.exact_grads(X, dY)
    assert dW.tolist() == [[1.0, 2.0], [6.0, 8.0]]
    assert db2.tolist() == [1.0, 2.0]


def test_no_bias_and_bias_shape():
    X, W, b, _ = _tiny(2)
    Y0, _ = rmm.forward(X, W, None, 2, sketch.RADEMACHER, 1, 1)
    Y1, _ = rmm.forward(X, W, b, 2, sketch.RADEMACHER, 1, 1)
    assert np.allclose(Y1 - Y0, np.broadcast_to(b, Y0.shape))


def test_estimator_two_ways():
    """dW_rmm = dY^T (S S^T) X (first line of Eq. 4) = (S^T dY)^T X_proj."""
    X, W, _, dY = _tiny(3, n=9, d_in=4, d_out=6)
    for kind in (sketch.GAUSSIAN, sketch.RADEMACHER):
        k, seed, off = 5, 77, 123456789012
        S = sketch.sketch_S(9, k, kind, seed, off)
        _, Xp = rmm.forward(X, W, None, k, kind, seed, off)
        _, dW, _ = rmm.backward(dY, W, Xp, kind, seed, off)
        assert np.allclose(dW, dY.T @ (S @ S.T) @ X, rtol=1e-12, atol=1e-12)
        assert np.allclose(Xp, rmm.sketch_apply(X, k, kind, seed, off))
        G = rmm.sketch_apply(dY, k, kind, seed, off)
        assert np.allclose(dW, G.T @ Xp, rtol=1e-12, atol=1e-12)


def test_backward_needs_the_forward_state():
    X, W, _, dY = _tiny(4, n=16)
    _, Xp = rmm.forward(X, W, None, 8, sketch.GAUSSIAN, 5, 0)
    _, dW_same, _ = rmm.backward(dY, W, Xp, sketch.GAUSSIAN, 5, 0)
    _, dW_other, _ = rmm.backward(dY, W, Xp, sketch.GAUSSIAN, 5, 1)
    assert not np.allclose(dW_same, dW_other)


def test_unbiased_monte_carlo():
    """Mean of dW_rmm over M independent states -> dY^T X, error ~ sqrt(Var/M)."""
    from oracle import variance
    X, W, _, dY = _tiny(5, n=8, d_in=3, d_out=2)
    dY = dY + 0.5 * X[:, :2]                       # correlated, so dY^T X is far from 0
    exact, _ = rmm.exact_grads(X, dY)
    k, M = 4, 8000
    for kind in (sketch.GAUSSIAN, sketch.RADEMACHER):
        acc = np.zeros_like(exact)
        for t in range(M):
            _, Xp = rmm.forward(X, W, None, k, kind, 2024, t)
            _, dW, _ = rmm.backward(dY, W, Xp, kind, 2024, t)
            acc += dW
        acc /= M
        for o in range(exact.shape[0]):
            for c in range(exact.shape[1]):
                sd = math.sqrt(variance.inner_product_variance(
                    dY[:, o], X[:, c], k, kind == sketch.RADEMACHER) / M)
                assert abs(acc[o, c] - exact[o, c]) < 5 * sd
        # a wrong normalisation (1/k or 1 instead of 1/sqrt(k)) would be off by >= 2x
        assert np.linalg.norm(acc - exact) < 0.1 * np.linalg.norm(exact)


def test_memory_and_flops_formulas():
    """Section 2.4.1: stored input shrinks by exactly k/N; Table 1 cost terms."""
    for n, d_in, d_out, k, e in ((4096, 768, 3072, 410, 2), (16384, 1024, 4096, 1638, 2), (256, 128, 128, 32, 4)):
        saved, plain = rmm.saved_bytes(n, d_in, k, e)
        assert (saved - 16) * n == plain * k
        f = rmm.flops(n, d_in, d_out, k)
        assert f["Y"] == f["dX"] == 2 * n * d_in * d_out
        assert f["X_proj"] == 2 * n * k * d_in                                 # forward extra: B B_proj N_in
        assert f["G"] + f["dW"] == 2 * k * d_out * (n + d_in)                   # backward: B_proj N_out (B + N_in)
    f = rmm.flops(4096, 768, 3072, 410)
    total = f["Y"] + f["X_proj"] + f["dX"] + f["G"] + f["dW"]
    assert abs(total / 1e9 - 53.5) < 0.05
