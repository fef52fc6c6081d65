"""GPU: parity on shapes chosen around every switch point of the host-side kernel selection
(streaming kernel up to k = 64, LDS-generated sketch tile from d = 1024, 256x256 tiles from 160
such tiles, two wave groups for few tiles with a contraction of 768 or more, token slices that
do not divide n) and on seeded random shapes."""
import math

import numpy as np
import pytest
import torch

import paper_2201_13195_amd as rmm
from paper_2201_13195_amd import synth
from oracle import rmm as o_rmm
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda"

BOUNDARY = [
    # (n, d_in, d_out, k)
    (700, 1016, 1024, 64), (700, 1024, 1032, 65), (1300, 1032, 1016, 63),   # sketch kernel switches (k, d)
    (2500, 264, 4096, 129), (2560, 4096, 256, 70),                            # 160 / 10 x 16 large tiles in Y / dX
    (2432, 264, 4096, 129),                                                   # 152 large tiles: small-tile path
    (260, 1536, 136, 1536), (260, 1528, 136, 1528),                           # long contractions, few tiles
    (1200, 768, 1024, 100), (1200, 760, 1024, 100),                           # 80 tiles of Y, contraction at / below 768
    (127, 520, 264, 127), (129, 520, 264, 130), (1, 1024, 1024, 1),           # token blocks of 128, n = 1
    (3000, 2056, 8, 410), (3000, 8, 2056, 410),                               # one 8-wide side
]


def random_shapes(count, seed):
    g = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        n = int(g.integers(1, 2600))
        d_in, d_out = (int(8 * g.integers(1, 200)) for _ in range(2))
        k = int(g.choice([g.integers(1, 65), g.integers(65, 700)]))
        out.append((n, d_in, d_out, k))
    return out


def rel_fro(got, want):
    return float(np.linalg.norm(synth.to_f64(got) - want) / max(np.linalg.norm(want), 1e-300))


@pytest.mark.parametrize("shape", BOUNDARY + random_shapes(16, 20260101))
def test_parity_on_switch_points_and_random_shapes(shape):
    n, d_in, d_out, k = shape
    kind = rmm.GAUSSIAN if (n + k) % 2 == 0 else rmm.RADEMACHER
    X, W, dY = synth.layer_inputs(n, d_in, d_out, "bf16", (n, d_in + 1, d_out + 2), w_std=1.0 / math.sqrt(d_in))
    seed, offset = 1234 + k, n
    Y, Xp = rmm.rmm_forward(X.to(DEV), W.to(DEV), None, k, kind, seed, offset)
    dX, dW, _ = rmm.rmm_backward(dY.to(DEV), W.to(DEV), Xp, kind, seed, offset)
    X64, W64, dY64 = synth.to_f64(X), synth.to_f64(W), synth.to_f64(dY)
    oY, oXp = o_rmm.forward(X64, W64, None, k, kind, seed, offset)
    odX, odW, _ = o_rmm.backward(dY64, W64, synth.to_f64(Xp), kind, seed, offset)
    errs = {"Y": rel_fro(Y, oY), "X_proj": rel_fro(Xp, oXp), "dX": rel_fro(dX, odX), "dW": rel_fro(dW, odW)}
    print(shape, kind, {k_: "%.2e" % v for k_, v in errs.items()}, flush=True)
    for name, e in errs.items():
        assert e <= 1e-2, (shape, name, e)
    for name, got, want in (("Y", Y, oY), ("X_proj", Xp, oXp), ("dX", dX, odX), ("dW", dW, odW)):
        assert_close(got, want, name, "bf16", str(shape))
