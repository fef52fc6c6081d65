"""Comparison helpers shared by the GPU parity tests (no test is collected from this file).

Two criteria, both against the fp64 oracle on identical inputs:

  * relative Frobenius error of the whole matrix, <= 1e-5 (fp32) / 1e-2 (bf16);
  * an entry-by-entry bound |got - want| <= RTOL * |want| + c * rms(want), which a run of wrong
    entries carrying a negligible share of the matrix's energy (one bad row, a bad tile edge)
    cannot pass: a wrong entry is off by about rms(want).

Where the constants come from (bf16: 8 significant bits, so one rounding is off by at most
u = 2^-8 relative, at the bottom of a binade, and by 0.0016 relative in the RMS).  RTOL counts the
roundings that act on the value as a whole when a single summand dominates it (n = 1 or k = 1 is
the extreme case): u for the output of Y and dX, 2u for X_proj (the generated entry, the output),
4u for dW (the generated entry, G, the output, and one u of margin).  The additive term covers
errors of the summands, which do not scale with the (possibly cancelling) sum but with its typical
size, rms(want):
  Y, dX      operands are exact, fp32 accumulation of <= 4096 products: c = 1e-3 is far above it;
  X_proj, G  every generated Gaussian entry is rounded to bf16 once, so a sum of n terms P_t x_t
             carries an error of standard deviation 0.0016 * rms; c = 1.2e-2 is 7.5 sigma
             (Rademacher entries are exact, the bound is then loose);
  dW         G is rounded to bf16 (0.0016) on top of its own summand errors (0.0016): 0.0023 * rms
             per entry of G and as much for the sum over k; c = 2e-2 is 8.7 sigma.
fp32: the generated Gaussian entries are within 4e-6 of the oracle's, sums of <= 4096 fp32
products add about 1e-6 * rms: RTOL = c = 2e-5 for every output.
"""
import numpy as np
import torch

from paper_2201_13195_amd import synth

FRO_TOL = {"f32": 1e-5, "bf16": 1e-2}
_U = 2.0 ** -8
RTOL = {
    "f32": {"Y": 2e-5, "dX": 2e-5, "X_proj": 2e-5, "dW": 2e-5, "db": 2e-5},
    "bf16": {"Y": _U, "dX": _U, "X_proj": 2 * _U, "dW": 4 * _U, "db": _U},
}
ATOL_RMS = {
    "f32": {"Y": 2e-5, "dX": 2e-5, "X_proj": 2e-5, "dW": 2e-5, "db": 2e-5},
    "bf16": {"Y": 1e-3, "dX": 1e-3, "X_proj": 1.2e-2, "dW": 2e-2, "db": 1e-3},
}


def as_f64(a):
    return synth.to_f64(a) if isinstance(a, torch.Tensor) else np.asarray(a, dtype=np.float64)


def rel_fro(got, want):
    got, want = as_f64(got), as_f64(want)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def elementwise_excess(got, want, what, dtype):
    """max over entries of |got - want| / (RTOL |want| + c rms(want)); <= 1 passes.
    Returns (excess, index of the worst entry)."""
    got, want = as_f64(got), as_f64(want)
    assert got.shape == want.shape, (got.shape, want.shape)
    rms = float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    bound = RTOL[dtype][what] * np.abs(want) + ATOL_RMS[dtype][what] * rms + 1e-300
    ratio = np.abs(got - want) / bound
    worst = int(np.argmax(ratio)) if ratio.size else 0
    return (float(ratio.flat[worst]) if ratio.size else 0.0), np.unravel_index(worst, want.shape) if ratio.size else ()


def assert_close(got, want, what, dtype, label=""):
    """Both criteria; returns the relative Frobenius error."""
    assert np.all(np.isfinite(as_f64(got))), (label, what, "non-finite output")
    fro = rel_fro(got, want)
    assert fro <= FRO_TOL[dtype], (label, what, "frobenius", fro)
    exc, where = elementwise_excess(got, want, what, dtype)
    assert exc <= 1.0, (label, what, "entry", where, "excess over the entry-wise bound", exc)
    return fro
