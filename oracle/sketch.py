"""The virtual sketch S (N x k) as a pure function of the saved PRNG state.

Test infrastructure.  The paper (Section 2.1, Eq. 5; Section 3.5) only says S
is drawn from a PRNG whose state is saved and replayed in the backward pass, with
E[S S^T] = I.  The element map below is this build's reading of that (the paper
is silent on it):

  state   = (seed, offset), two 64-bit integers
  key     = (seed mod 2^32, seed div 2^32)
  counter = (c0, j, offset mod 2^32, offset div 2^32)        j = sketch column

  Gaussian    c0 = i div 8.  The call's four words r0..r3 serve tokens
              8*c0 .. 8*c0+7 of column j, two tokens per word:
              w = r[(i mod 8) div 2], u1 = ((w div 2^16) + 1/2) / 2^16 in (0,1),
              u2 = (w mod 2^16) / 2^16 in [0,1); Box-Muller:
              P[i,j] = sqrt(-2 ln u1) * (cos(2 pi u2) if i even else sin(2 pi u2)).
  Rademacher  c0 = i div 128, t = i mod 128,
              bit = (r[t div 32] >> (t mod 32)) & 1,  P[i,j] = 1 - 2*bit.

  S = P / sqrt(k)   (Eq. 5; "proper normalization" of Section 3.5 for Rademacher).

  SORS        Subsampled orthonormal matrix with random signs (Section 2.1 names the
              family and gives no construction; Section 3.5 and the future-work paragraph
              only say that such S allow O(B N log B) products).  PARITY UNPINNED against
              the paper: the construction below is this build's own, the textbook
              subsampled randomized Hadamard transform:
                n_pad   = smallest power of two >= n
                sigma_i = the Rademacher entry of token i in column 0xFFFFFFFF
                r_j     = word (j mod 4) of the call with counter
                          (j div 4, 0xFFFFFFFE, offset) AND (n_pad - 1): a row of the
                          n_pad x n_pad Walsh-Hadamard matrix, drawn uniformly and
                          independently for every sketch column (with replacement)
                P[i,j]  = sigma_i * (-1)^popcount(i AND r_j)
              i.e. S^T A = sqrt(n_pad / k) * R H D [A; 0] with D = diag(sigma), H the
              orthonormal Walsh-Hadamard matrix (entries +-1/sqrt(n_pad), Sylvester
              order) and R the selection of rows r_0 .. r_{k-1}; E[R^T R] = (k/n_pad) I
              gives E[S S^T] = I.  Unlike the other kinds P depends on n (through n_pad).
"""
import numpy as np

from .philox import philox4x32_10

GAUSSIAN = 0
RADEMACHER = 1
SORS = 2

SORS_SIGN_COLUMN = 0xFFFFFFFF   # counter word 1 of the calls behind the token signs
SORS_ROW_COLUMN = 0xFFFFFFFE    # counter word 1 of the calls behind the selected rows


def _key_and_tail(seed, offset):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    offset = int(offset) & 0xFFFFFFFFFFFFFFFF
    return (seed & 0xFFFFFFFF, seed >> 32, offset & 0xFFFFFFFF, offset >> 32)


def words(n, k, kind, seed, offset):
    """Raw Philox words behind the sketch: uint32 array of shape (calls, k, 4),
    calls = ceil(n/8) (Gaussian) or ceil(n/128) (Rademacher); entry [c, j] is the
    call with counter (c, j, offset_lo, offset_hi)."""
    per_call = 8 if kind == GAUSSIAN else 128
    calls = -(-int(n) // per_call)
    k0, k1, o0, o1 = _key_and_tail(seed, offset)
    c0 = np.arange(calls, dtype=np.uint64)[:, None]
    c1 = np.arange(int(k), dtype=np.uint64)[None, :]
    r = philox4x32_10(c0, c1, o0, o1, k0, k1)
    return np.stack(r, axis=-1)


def rademacher_bits(n, k, seed, offset):
    """uint8 (n, k): the sign bit behind each Rademacher entry (1 -> P = -1)."""
    n, k = int(n), int(k)
    w = words(n, k, RADEMACHER, seed, offset)                       # (calls, k, 4)
    shifts = np.arange(32, dtype=np.uint32)
    bits = (w[..., None] >> shifts) & np.uint32(1)                  # (calls, k, 4, 32): bit b of word q
    bits = bits.reshape(w.shape[0], k, 128)                         # t = 32*q + b
    return bits.transpose(0, 2, 1).reshape(-1, k)[:n].astype(np.uint8)   # row i = 128*call + t


def sors_padded_length(n):
    """Smallest power of two >= n (n >= 1)."""
    n = int(n)
    p = 1
    while p < n:
        p *= 2
    return p


def sors_signs(n, seed, offset):
    """float64 (n,): sigma_i = +-1, the Rademacher map applied to column 0xFFFFFFFF."""
    n = int(n)
    k0, k1, o0, o1 = _key_and_tail(seed, offset)
    calls = -(-n // 128)
    r = philox4x32_10(np.arange(calls, dtype=np.uint64), SORS_SIGN_COLUMN, o0, o1, k0, k1)
    w = np.stack(r, axis=-1)                                        # (calls, 4)
    bits = (w[..., None] >> np.arange(32, dtype=np.uint32)) & np.uint32(1)
    return 1.0 - 2.0 * bits.reshape(-1)[:n].astype(np.float64)      # token i = 128*call + 32*word + bit


def sors_rows(n, k, seed, offset):
    """int64 (k,): the Walsh-Hadamard row r_j behind sketch column j, uniform on [0, n_pad)."""
    k = int(k)
    k0, k1, o0, o1 = _key_and_tail(seed, offset)
    calls = -(-k // 4)
    r = philox4x32_10(np.arange(calls, dtype=np.uint64), SORS_ROW_COLUMN, o0, o1, k0, k1)
    w = np.stack(r, axis=-1).reshape(-1)[:k].astype(np.int64)       # column j = 4*call + word
    return w & (sors_padded_length(n) - 1)


def hadamard_sign(i, r):
    """(-1)^popcount(i AND r): entry (r, i) of the unnormalised Walsh-Hadamard matrix in
    Sylvester order (H_1 = [1], H_2m = [[H_m, H_m], [H_m, -H_m]]).  Broadcasts."""
    x = np.bitwise_and(np.asarray(i, dtype=np.int64), np.asarray(r, dtype=np.int64))
    parity = np.zeros_like(x)
    while np.any(x):
        parity ^= x & 1
        x = x >> 1
    return 1.0 - 2.0 * parity.astype(np.float64)


def sketch_P(n, k, kind, seed, offset):
    """Unscaled sketch P (n x k, float64): unit-variance Gaussian or +-1 entries."""
    n, k = int(n), int(k)
    if kind == SORS:
        sigma = sors_signs(n, seed, offset)
        rows = sors_rows(n, k, seed, offset)
        return sigma[:, None] * hadamard_sign(np.arange(n)[:, None], rows[None, :])
    if kind == RADEMACHER:
        return 1.0 - 2.0 * rademacher_bits(n, k, seed, offset).astype(np.float64)
    if kind != GAUSSIAN:
        raise ValueError("unknown sketch kind")
    w = words(n, k, GAUSSIAN, seed, offset).astype(np.uint64)       # (calls, k, 4)
    u1 = ((w >> np.uint64(16)).astype(np.float64) + 0.5) / 65536.0  # (0, 1)
    u2 = (w & np.uint64(0xFFFF)).astype(np.float64) / 65536.0       # [0, 1)
    rad = np.sqrt(-2.0 * np.log(u1))
    ang = 2.0 * np.pi * u2
    pair = np.stack((rad * np.cos(ang), rad * np.sin(ang)), axis=-1)   # (calls, k, 4, 2): word q -> tokens 2q, 2q+1
    pair = pair.reshape(w.shape[0], k, 8)
    return np.ascontiguousarray(pair.transpose(0, 2, 1).reshape(-1, k)[:n])  # row i = 8*call + slot


def sketch_S(n, k, kind, seed, offset):
    """S = P / sqrt(k): entries of variance 1/k so that E[S S^T] = I_N (Eq. 5)."""
    return sketch_P(n, k, kind, seed, offset) / np.sqrt(float(k))
