"""Pins for oracle.variance: the paper's B = 2 worked example (Section 2.3),
Monte-Carlo variance of the estimate on correlated inputs (decides the sign in
Lemma 2.2 and the Rademacher correction), the 1/k decay, a chi-square special
case, Theorem 2.3's bound, and pins of Lemma 2.1 and of alpha that do not vanish (hand
cases with X^T Y != 0, the definition the lemma's proof starts from, a row-sampling Monte-Carlo)."""
import math
import os

import numpy as np

from oracle import rmm, sketch, variance


def test_worked_example(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "worked_example_b2.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([float(t) for t in line.split()])
    assert len(rows) >= 3
    for eps, sgd, rmm_val in rows:
        X = np.array([[1.0, 0.0], [-eps, 0.0]])
        Y = np.array([[1.0, 0.0], [1.0 / eps, 0.0]])
        assert np.allclose(X.T @ Y, 0.0, atol=1e-15)
        assert math.isclose((2 - 1) * variance.d2_sgd(X, Y), sgd, rel_tol=1e-12)
        for kproj in (1, 3, 10):
            # X^T Y = 0, so the printed and the corrected form coincide here
            assert math.isclose(kproj * variance.d2_rmm_printed(X, Y, kproj), rmm_val, rel_tol=1e-12)
            assert math.isclose(kproj * variance.rmm_variance_gaussian(Y, X, kproj), rmm_val, rel_tol=1e-12)
        assert variance.alpha(X, Y) < 1e-30


def test_single_column_is_chi_square():
    """X = Y = a (one column): a^T S S^T a = |a|^2 chi2_k / k, variance 2|a|^4/k.
    The printed lemma would give 0 here."""
    a = np.array([[1.0], [2.0], [-0.5]])
    k = 7
    want = 2.0 * float(np.sum(a * a)) ** 2 / k
    assert math.isclose(variance.rmm_variance_gaussian(a, a, k), want, rel_tol=1e-12)
    assert math.isclose(variance.inner_product_variance(a[:, 0], a[:, 0], k), want, rel_tol=1e-12)
    assert variance.d2_rmm_printed(a, a, k) == 0.0


def test_frobenius_form_is_sum_of_entry_forms():
    g = np.random.default_rng(3)
    X, Y = g.standard_normal((6, 3)), g.standard_normal((6, 2))
    for rad in (False, True):
        tot = sum(variance.inner_product_variance(Y[:, p], X[:, q], 5, rad)
                  for p in range(2) for q in range(3))
        f = variance.rmm_variance_rademacher if rad else variance.rmm_variance_gaussian
        assert math.isclose(f(X, Y, 5), tot, rel_tol=1e-12)


def _mc_variance(X, dY, k, kind, M, seed):
    exact, _ = rmm.exact_grads(X, dY)
    W = np.zeros((dY.shape[1], X.shape[1]))
    err2 = np.empty(M)
    for t in range(M):
        _, Xp = rmm.forward(X, W, None, k, kind, seed, t)
        _, dW, _ = rmm.backward(dY, W, Xp, kind, seed, t)
        err2[t] = np.sum((dW - exact) ** 2)
    return err2.mean(), err2.std(ddof=1) / math.sqrt(M)


def test_monte_carlo_variance_on_correlated_inputs():
    g = np.random.default_rng(11)
    X = g.standard_normal((8, 3))
    dY = 0.8 * X[:, :2] + 0.3 * g.standard_normal((8, 2))      # strongly correlated with X
    k, M = 4, 12000
    vg = variance.rmm_variance_gaussian(X, dY, k)
    vr = variance.rmm_variance_rademacher(X, dY, k)
    vp = variance.d2_rmm_printed(X, dY, k)
    assert vp < 0.75 * vg and vr < 0.9 * vg                     # the three candidates are well apart
    mc_g, se_g = _mc_variance(X, dY, k, sketch.GAUSSIAN, M, 31)
    mc_r, se_r = _mc_variance(X, dY, k, sketch.RADEMACHER, M, 32)
    assert abs(mc_g - vg) < 5 * se_g and abs(mc_g - vg) < 0.08 * vg
    assert abs(mc_r - vr) < 5 * se_r and abs(mc_r - vr) < 0.08 * vr
    assert abs(mc_g - vp) > 10 * se_g                            # minus sign of the printed lemma is excluded
    assert abs(mc_r - vg) > 10 * se_r                            # Rademacher needs its correction


def test_error_decays_like_inverse_sqrt_k():
    """Section 2.2: RMS error ~ k^-1/2, i.e. mean squared error ~ 1/k."""
    g = np.random.default_rng(12)
    X, dY = g.standard_normal((16, 3)), g.standard_normal((16, 2))
    m4, _ = _mc_variance(X, dY, 4, sketch.GAUSSIAN, 4000, 41)
    m16, _ = _mc_variance(X, dY, 16, sketch.GAUSSIAN, 4000, 42)
    slope = math.log(math.sqrt(m16 / m4)) / math.log(16 / 4)
    assert abs(slope + 0.5) < 0.05


def test_theorem_bound_with_printed_lemma():
    """Theorem 2.3 as stated (with the lemma's printed form):
    k/(B-1) * D2_RMM / D2_SGD <= (alpha+1)/alpha."""
    g = np.random.default_rng(13)
    for _ in range(20):
        X, Y = g.standard_normal((12, 4)), g.standard_normal((12, 5))
        k = 6
        a = variance.alpha(X, Y)
        assert 0.0 <= a <= 1.0
        lhs = k / (12 - 1) * variance.d2_rmm_printed(X, Y, k) / variance.d2_sgd(X, Y)
        assert lhs <= (a + 1) / a


def _hand_cases(golden_dir):
    cases = []
    with open(os.path.join(golden_dir, "variance_hand_cases.txt")) as f:
        for line in f:
            if not line.strip() or line.startswith("#"):
                continue
            t = [float(v) for v in line.split()]
            B, N, M = int(t[0]), int(t[1]), int(t[2])
            X = np.array(t[3:3 + B * N]).reshape(B, N)
            Y = np.array(t[3 + B * N:3 + B * N + B * M]).reshape(B, M)
            cases.append((X, Y, t[-2], t[-1]))
    assert len(cases) >= 4
    return cases


def test_hand_cases_with_nonzero_cross_term(golden_dir):
    """Lemma 2.1 and Theorem 2.3's alpha on integer inputs worked out by hand, where the
    |X^T Y|^2 term does not vanish (in the paper's own example it does)."""
    for X, Y, want_sgd, want_alpha in _hand_cases(golden_dir):
        assert np.any(X.T @ Y != 0.0)
        assert math.isclose(variance.d2_sgd(X, Y), want_sgd, rel_tol=1e-13, abs_tol=1e-13)
        assert math.isclose(variance.alpha(X, Y), want_alpha, rel_tol=1e-13)


def test_d2_sgd_is_the_sample_variance_of_the_mean():
    """The definition Lemma 2.1's proof starts from: Z_k = B x_k y_k^T has mean X^T Y, and
    D2_SGD = 1/(B(B-1)) sum_k |Z_k - X^T Y|_F^2 (unbiased sample variance of Z, over B)."""
    g = np.random.default_rng(21)
    for B, N, M in ((2, 3, 2), (5, 4, 3), (9, 2, 6)):
        X, Y = g.standard_normal((B, N)), 0.5 * g.standard_normal((B, M)) + 0.7
        zbar = X.T @ Y
        tot = 0.0
        for kk in range(B):
            Z = B * np.outer(X[kk], Y[kk])
            tot += float(np.sum((Z - zbar) ** 2))
        assert math.isclose(variance.d2_sgd(X, Y), tot / (B * (B - 1)), rel_tol=1e-12)


def test_d2_sgd_against_row_sampling_monte_carlo():
    """Lemma 2.1 estimates the noise of a gradient formed from randomly selected samples.  Draw B
    rows with replacement from the B given ones: the mean of Z = B x y^T over the draw has
    expectation X^T Y and mean squared deviation (population variance of Z) / B, which is
    (B-1)/B * D2_SGD.  Inputs are correlated so that the cross term is a large part of the value."""
    g = np.random.default_rng(22)
    B = 6
    X = g.standard_normal((B, 3)) + 1.0
    Y = 0.6 * X[:, :2] + 0.2 * g.standard_normal((B, 2))
    rows = float(np.sum(np.sum(X * X, axis=1) * np.sum(Y * Y, axis=1)))
    assert np.sum((X.T @ Y) ** 2) > 0.25 * B * rows         # the cross term matters here
    M = 200000
    idx = g.integers(0, B, size=(M, B))
    Zk = B * np.einsum("kn,km->knm", X, Y)                   # per-sample matrices
    means = Zk[idx].mean(axis=1)                             # (M, N, M')
    err2 = np.sum((means - (X.T @ Y)[None]) ** 2, axis=(1, 2))
    mc, se = err2.mean(), err2.std(ddof=1) / math.sqrt(M)
    want = (B - 1) / B * variance.d2_sgd(X, Y)
    assert abs(mc - want) < 5 * se and abs(mc - want) < 0.02 * want
    # dropping the cross term, flipping its sign or halving it is far outside the Monte-Carlo error
    cross = float(np.sum((X.T @ Y) ** 2)) / (B - 1.0) * (B - 1) / B
    assert 0.5 * cross > 20 * se


def test_alpha_special_cases():
    """Theorem 2.3's alpha = |X^T Y|^2 / (|X|^2 |Y|^2): 1 for X = Y = one column, 0 for orthogonal
    columns, cos^2 of the angle for two single columns, invariant under scaling of X and of Y."""
    a = np.array([[1.0], [2.0], [-0.5]])
    assert math.isclose(variance.alpha(a, a), 1.0, rel_tol=1e-14)
    assert variance.alpha(np.array([[1.0], [1.0]]), np.array([[1.0], [-1.0]])) == 0.0
    u, v = np.array([[1.0], [0.0]]), np.array([[1.0], [1.0]])
    assert math.isclose(variance.alpha(u, v), 0.5, rel_tol=1e-14)
    g = np.random.default_rng(23)
    X, Y = g.standard_normal((7, 3)), g.standard_normal((7, 4))
    assert math.isclose(variance.alpha(3.0 * X, -0.25 * Y), variance.alpha(X, Y), rel_tol=1e-12)
    # entry-wise statement: sum over pairs of columns of squared inner products, over the product of norms
    tot = sum(float(X[:, p] @ Y[:, q]) ** 2 for p in range(3) for q in range(4))
    assert math.isclose(variance.alpha(X, Y), tot / (float(np.sum(X * X)) * float(np.sum(Y * Y))), rel_tol=1e-12)
