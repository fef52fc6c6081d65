"""GPU statistical checks of the estimate dW = (S^T dY)^T X_proj over many sketch
states: unbiasedness (Eq. 4) and the closed-form variance (Lemma 2.2 with the
corrected sign, and the Rademacher correction)."""
import math

import numpy as np
import pytest
import torch

import paper_2201_13195_amd as rmm
from paper_2201_13195_amd import synth
from oracle import rmm as o_rmm
from oracle import variance as o_var

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _errors_over_states(X, W, dY, k, kind, seed, states):
    Xd, Wd, dYd = X.to(DEV), W.to(DEV), dY.to(DEV)
    exact, _ = o_rmm.exact_grads(synth.to_f64(X), synth.to_f64(dY))
    exact_d = torch.from_numpy(exact).to(DEV)
    mean = torch.zeros_like(exact_d)
    err2_d = torch.zeros(states, dtype=torch.float64, device=DEV)
    for t in range(states):
        _, Xp = rmm.rmm_forward(Xd, Wd, None, k, kind, seed, t)
        _, dW, _ = rmm.rmm_backward(dYd, Wd, Xp, kind, seed, t, need_dX=False)
        dW64 = dW.to(torch.float64)
        mean += dW64
        err2_d[t] = torch.sum((dW64 - exact_d) ** 2)
    mean /= states
    err2 = err2_d.cpu().numpy()
    return exact, mean.cpu().numpy(), err2.mean(), err2.std(ddof=1) / math.sqrt(states)


def test_thousand_state_variance_at_base_shape():
    """N = 4096, d = 768, k = 410, fixed X and dY, 1000 sketch states."""
    n, d, k, states = 4096, 768, 410, 1000
    X, W, dY = synth.layer_inputs(n, d, d, "bf16", (5901, 5903, 5902))
    exact, mean, mc, se = _errors_over_states(X, W, dY, k, rmm.GAUSSIAN, 0x5EED0005, states)
    want = o_var.rmm_variance_gaussian(synth.to_f64(X), synth.to_f64(dY), k)
    print("variance: monte-carlo %.6e +- %.1e, closed form %.6e" % (mc, se, want), flush=True)
    assert abs(mc - want) < max(5 * se, 0.01 * want)
    # unbiased: the mean's error shrinks like sqrt(variance / states)
    assert np.linalg.norm(mean - exact) < 1.5 * math.sqrt(want / states)


@pytest.mark.parametrize("kind", [rmm.GAUSSIAN, rmm.RADEMACHER])
def test_variance_on_correlated_low_rank_inputs(kind):
    """Inputs where |dY^T X|^2 and sum_i |x_i|^2 |dy_i|^2 are a large part of
    |X|^2 |dY|^2, so a wrong sign or a missing Rademacher term is visible."""
    n, d_in, d_out, k, states = 512, 64, 48, 32, 20000
    g = np.random.default_rng(77)
    a = g.standard_normal((n, 2)) * np.array([3.0, 1.0])
    a[:8] *= 6.0                                           # a few heavy rows: Rademacher term matters
    X = synth.to_torch(a @ g.standard_normal((2, d_in)) + 0.05 * g.standard_normal((n, d_in)), "f32")
    dY = synth.to_torch(a @ g.standard_normal((2, d_out)) + 0.05 * g.standard_normal((n, d_out)), "f32")
    W = synth.to_torch(g.standard_normal((d_out, d_in)), "f32")
    X64, dY64 = synth.to_f64(X), synth.to_f64(dY)
    vg = o_var.rmm_variance_gaussian(X64, dY64, k)
    vr = o_var.rmm_variance_rademacher(X64, dY64, k)
    vp = o_var.d2_rmm_printed(X64, dY64, k)
    assert vp < 0.7 * vg and vr < 0.93 * vg
    exact, mean, mc, se = _errors_over_states(X, W, dY, k, kind, 99, states)
    want = vg if kind == rmm.GAUSSIAN else vr
    print("kind %d: monte-carlo %.5e +- %.1e, closed form %.5e (other candidates %.5e %.5e)"
          % (kind, mc, se, want, vp, vg if kind == rmm.RADEMACHER else vr), flush=True)
    assert abs(mc - want) < 5 * se
    assert abs(mc - want) < 0.05 * want
    other = vg if kind == rmm.RADEMACHER else vr
    assert abs(mc - other) > 4 * se and abs(mc - vp) > 20 * se
    assert np.linalg.norm(mean - exact) < 5 * math.sqrt(want / states)
