"""Pins for the SORS sketch of oracle.sketch (Section 2.1 names the family; the construction,
a subsampled randomized Walsh-Hadamard transform, is this build's own, so parity with the
paper is unpinned).  What is pinned here is the construction itself: the Hadamard entries
against scipy's Sylvester matrix and the recursive definition, orthonormality, the sign and
row streams against the plain-int generator, E[S S^T] = I by exact enumeration of the rows,
the fast-transform identity S^T A = sqrt(n_pad/k) R H D A, and unbiasedness of the estimator."""
import numpy as np
import scipy.linalg

from oracle import rmm as o_rmm
from oracle import sketch
from oracle.philox import philox4x32_10_scalar

SEED = 0x0F1E2D3C4B5A6978
OFFSET = (3 << 32) | 11


def test_hadamard_sign_is_the_sylvester_matrix():
    for m in (1, 2, 8, 64, 256):
        idx = np.arange(m)
        H = sketch.hadamard_sign(idx[None, :], idx[:, None])
        assert np.array_equal(H, scipy.linalg.hadamard(m).astype(np.float64))
        assert np.array_equal(H @ H.T, m * np.eye(m))          # rows orthogonal, norm sqrt(m)
    # the recursion H_2m = [[H_m, H_m], [H_m, -H_m]] written out
    H4 = sketch.hadamard_sign(np.arange(4)[None, :], np.arange(4)[:, None])
    H8 = sketch.hadamard_sign(np.arange(8)[None, :], np.arange(8)[:, None])
    assert np.array_equal(H8, np.block([[H4, H4], [H4, -H4]]))


def test_padded_length():
    assert [sketch.sors_padded_length(n) for n in (1, 2, 3, 4, 5, 127, 128, 129, 4096, 4097)] == \
        [1, 2, 4, 4, 8, 128, 128, 256, 4096, 8192]


def test_sign_and_row_streams_against_the_plain_int_generator():
    key = (SEED & 0xFFFFFFFF, SEED >> 32)
    tail = (OFFSET & 0xFFFFFFFF, OFFSET >> 32)
    n, k = 300, 23
    sig = sketch.sors_signs(n, SEED, OFFSET)
    rows = sketch.sors_rows(n, k, SEED, OFFSET)
    for i in range(n):
        r = philox4x32_10_scalar((i // 128, 0xFFFFFFFF) + tail, key)
        t = i % 128
        assert sig[i] == 1.0 - 2.0 * ((r[t // 32] >> (t % 32)) & 1)
    for j in range(k):
        r = philox4x32_10_scalar((j // 4, 0xFFFFFFFE) + tail, key)
        assert rows[j] == r[j % 4] & 511                      # n_pad = 512
    # the signs are the Rademacher map's column 0xFFFFFFFF: same bits as that map gives any column
    # when called with the same counter
    assert set(np.unique(sig)) <= {-1.0, 1.0}
    assert abs(sketch.sors_signs(1 << 16, SEED, OFFSET).mean()) < 4.0 / 256      # balanced: 4 sigma of 2^-8


def test_rows_are_uniform():
    n, k = 1 << 10, 1 << 16
    rows = sketch.sors_rows(n, k, SEED, OFFSET)
    assert rows.min() >= 0 and rows.max() < n
    counts = np.bincount(rows, minlength=n)                    # expectation 64 per row
    chi2 = ((counts - 64.0) ** 2 / 64.0).sum()                 # 1023 degrees of freedom, sd ~ 45
    assert abs(chi2 - 1023.0) < 5 * 45.3


def test_entry_definition_and_value_set():
    n, k = 77, 9
    P = sketch.sketch_P(n, k, sketch.SORS, SEED, OFFSET)
    sig = sketch.sors_signs(n, SEED, OFFSET)
    rows = sketch.sors_rows(n, k, SEED, OFFSET)
    for i in range(n):
        for j in range(k):
            assert P[i, j] == sig[i] * (-1.0) ** bin(i & int(rows[j])).count("1")
    assert np.array_equal(np.abs(P), np.ones((n, k)))


def test_expectation_of_s_st_is_the_identity_by_enumeration():
    """E over the row draw, exactly: every column picks each of the n_pad rows with probability
    1/n_pad, so E[S S^T] = (1/k) * k * (1/n_pad) * sum_r p_r p_r^T with p_r = D h_r restricted
    to the first n tokens; the sum over all rows of the Hadamard matrix is n_pad * I."""
    for n in (16, 24, 100):
        n_pad = sketch.sors_padded_length(n)
        sig = sketch.sors_signs(n, SEED, OFFSET)
        acc = np.zeros((n, n))
        for r in range(n_pad):
            p = sig * sketch.hadamard_sign(np.arange(n), r)
            acc += np.outer(p, p)
        assert np.array_equal(acc / n_pad, np.eye(n))


def test_equals_the_transform_form():
    """S^T A = sqrt(n_pad / k) * R H D [A; 0] with the orthonormal Hadamard matrix from scipy."""
    rng = np.random.default_rng(5)
    for n, k, d in ((64, 10, 7), (100, 33, 5), (1, 3, 4)):
        A = rng.standard_normal((n, d))
        n_pad = sketch.sors_padded_length(n)
        S = sketch.sketch_S(n, k, sketch.SORS, SEED, OFFSET)
        Apad = np.zeros((n_pad, d))
        Apad[:n] = sketch.sors_signs(n, SEED, OFFSET)[:, None] * A
        T = (scipy.linalg.hadamard(n_pad) / np.sqrt(n_pad)) @ Apad if n_pad > 1 else Apad
        want = np.sqrt(n_pad / k) * T[sketch.sors_rows(n, k, SEED, OFFSET)]
        assert np.allclose(S.T @ A, want, rtol=1e-12, atol=1e-12)


def test_distinct_rows_give_orthogonal_columns_when_n_is_a_power_of_two():
    n, k = 128, 40
    P = sketch.sketch_P(n, k, sketch.SORS, SEED, OFFSET)
    rows = sketch.sors_rows(n, k, SEED, OFFSET)
    G = P.T @ P
    for a in range(k):
        for b in range(k):
            assert G[a, b] == (n if rows[a] == rows[b] else 0.0)


def test_depends_on_state_and_on_n_only_through_the_padded_length():
    a = sketch.sketch_P(100, 8, sketch.SORS, SEED, OFFSET)
    assert np.array_equal(a, sketch.sketch_P(128, 8, sketch.SORS, SEED, OFFSET)[:100])   # same n_pad
    assert not np.array_equal(a, sketch.sketch_P(100, 8, sketch.SORS, SEED + 1, OFFSET))
    assert not np.array_equal(a, sketch.sketch_P(100, 8, sketch.SORS, SEED, OFFSET + 1))
    assert np.array_equal(a[:, :5], sketch.sketch_P(100, 5, sketch.SORS, SEED, OFFSET))  # prefix in k


def test_weight_gradient_is_unbiased_with_the_sors_sketch():
    """Monte-Carlo over states: the mean of dW_hat = (S^T dY)^T (S^T X) approaches dY^T X
    at the 1/sqrt(trials) rate (Section 2.1's requirement E[S S^T] = I is all it needs)."""
    rng = np.random.default_rng(11)
    n, d_in, d_out, k, trials = 48, 5, 4, 12, 6000
    X = rng.standard_normal((n, d_in))
    dY = rng.standard_normal((n, d_out))
    exact = dY.T @ X
    acc = np.zeros_like(exact)
    sq = np.zeros_like(exact)
    for t in range(trials):
        S = sketch.sketch_S(n, k, sketch.SORS, SEED, t)
        est = (S.T @ dY).T @ (S.T @ X)
        acc += est
        sq += est * est
    mean = acc / trials
    sd = np.sqrt(np.maximum(sq / trials - mean * mean, 0.0) / trials)
    assert np.all(np.abs(mean - exact) < 5.0 * sd + 1e-12)
    # the layer oracle takes the kind like the other two
    S = sketch.sketch_S(n, k, sketch.SORS, SEED, 0)
    W = rng.standard_normal((d_out, d_in))
    Y, X_proj = o_rmm.forward(X, W, None, k, sketch.SORS, SEED, 0)
    assert np.allclose(X_proj, S.T @ X) and np.allclose(Y, X @ W.T)
    dX, dW, db = o_rmm.backward(dY, W, X_proj, sketch.SORS, SEED, 0)
    assert np.allclose(dW, (S.T @ dY).T @ X_proj) and np.allclose(dX, dY @ W)
