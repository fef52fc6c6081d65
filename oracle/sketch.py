"""The virtual sketch S (N x k) as a pure function of the saved PRNG state.

Test infrastructure.  The paper (Section 2.1, Eq. 5; Section 3.4) only says S
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

  S = P / sqrt(k)   (Eq. 5; "proper normalization" of Section 3.4 for Rademacher).
"""
import numpy as np

from .philox import philox4x32_10

GAUSSIAN = 0
RADEMACHER = 1


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


def sketch_P(n, k, kind, seed, offset):
    """Unscaled sketch P (n x k, float64): unit-variance Gaussian or +-1 entries."""
    n, k = int(n), int(k)
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
