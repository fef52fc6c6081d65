"""GPU: an operand of more than 2^31 bytes (X of 2^31 + 2^18 bytes) stays on the MFMA kernels, whose
32-bit buffer offsets are relative to the rows a work-group reads, and matches the oracle: Y and dX
on sampled rows (they are row-wise independent), X_proj and dW in full, with the oracle's S applied
to X in row blocks.  k = 8 takes the streaming sketch kernel, k = 72 the tiled one."""
import numpy as np
import pytest
import torch

import paper_2201_13195_amd as rmm
from paper_2201_13195_amd import synth
from oracle import sketch as o_sketch

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("k", [8, 72])
def test_operand_beyond_two_gib(k):
    n, d_in, d_out = (1 << 20) + 128, 1024, 8
    kind, seed, offset = rmm.RADEMACHER, 77, 3
    assert n * d_in * 2 >= 1 << 31
    block = 1 << 16
    X = torch.empty((n, d_in), dtype=torch.bfloat16, device=DEV)
    for r0 in range(0, n, block):
        rows = min(block, n - r0)
        X[r0:r0 + rows] = torch.from_numpy(synth.pattern_rows(r0, rows, d_in, 131, 17)).to(torch.bfloat16).to(DEV)
    W64 = synth.pattern_rows(0, d_out, d_in, 29, 13) / 16.0
    dY64 = synth.pattern_rows(0, n, d_out, 53, 11)
    W, dY = (torch.from_numpy(a).to(torch.bfloat16).to(DEV) for a in (W64, dY64))
    assert rmm.rmm_workspace_bytes(n, d_in, d_out, k, torch.bfloat16, kind, 0) > 0       # token slices: the MFMA path
    Y, Xp = rmm.rmm_forward(X, W, None, k, kind, seed, offset)
    dX, dW, _ = rmm.rmm_backward(dY, W, Xp, kind, seed, offset)
    torch.cuda.synchronize()

    S = o_sketch.sketch_S(n, k, kind, seed, offset)                     # n x k, fp64
    oXp = np.zeros((k, d_in))
    for r0 in range(0, n, block):
        rows = min(block, n - r0)
        oXp += S[r0:r0 + rows].T @ synth.pattern_rows(r0, rows, d_in, 131, 17)
    odW = (dY64.T @ S) @ synth.to_f64(Xp)

    def rel(a, b):
        return float(np.linalg.norm(a - b) / np.linalg.norm(b))

    sample = np.concatenate([np.arange(0, 300), np.arange(n // 2, n // 2 + 300), np.arange(n - 300, n)])
    Xs = np.concatenate([synth.pattern_rows(0, 300, d_in, 131, 17), synth.pattern_rows(n // 2, 300, d_in, 131, 17),
                         synth.pattern_rows(n - 300, 300, d_in, 131, 17)])
    errs = {"Y": rel(synth.to_f64(Y[sample]), Xs @ W64.T), "dX": rel(synth.to_f64(dX[sample]), dY64[sample] @ W64),
            "X_proj": rel(synth.to_f64(Xp), oXp), "dW": rel(synth.to_f64(dW), odW)}
    print({k_: "%.2e" % v for k_, v in errs.items()}, flush=True)
    for name, e in errs.items():
        assert e <= 1e-2, (name, e)
