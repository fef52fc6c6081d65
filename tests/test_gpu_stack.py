"""GPU: the 24-block stack of RoBERTa-large-shaped RMM linears (144 layers, N = 16384, k = 1638)
with every X_proj resident between the forward sweep and the reverse-order backward sweep.
Parity against the fp64 oracle on the first, middle and last layer of each of the three shapes
(with their own sketch states), and for the whole stack: finite outputs, run-to-run determinism
and the stored-activation bytes (Section 2.4.1: X_proj + 16 bytes of state per layer)."""
import numpy as np
import pytest
import torch

import paper_2201_13195_amd as rmm
from paper_2201_13195_amd import synth
from oracle import rmm as o_rmm
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda"


def rel_fro(got, want):
    return float(np.linalg.norm(synth.to_f64(got) - want) / max(np.linalg.norm(want), 1e-300))


def run_stack(layers, pool, keep):
    """Forward sweep keeping only X_proj and the state, then the backward sweep in reverse order.
    Returns X_proj per layer, the outputs of the layers in `keep`, and the two sweep times (ms)."""
    k, n = synth.STACK["k"], synth.STACK["n"]
    ws_bytes = 16
    for L in layers:
        for op in (0, 1):
            ws_bytes = max(ws_bytes, rmm.rmm_workspace_bytes(n, L["d_in"], L["d_out"], k, torch.bfloat16, rmm.GAUSSIAN, op))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    scratch = {}

    def buf(name, shape):
        key = (name,) + tuple(shape)
        if key not in scratch:
            scratch[key] = torch.empty(shape, dtype=torch.bfloat16, device=DEV)
        return scratch[key]

    xproj, kept = [None] * len(layers), {}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    torch.cuda.synchronize()
    ev[0].record()
    for L in layers:
        X, W, _ = pool[(L["shape"], L["pool"])]
        Y = buf("Y", (n, L["d_out"]))
        xproj[L["layer"]] = torch.empty((k, L["d_in"]), dtype=torch.bfloat16, device=DEV)
        rmm.rmm_forward(X, W, None, k, rmm.GAUSSIAN, L["seed"], L["offset"], Y=Y, X_proj=xproj[L["layer"]], ws=ws)
        if L["layer"] in keep:
            kept[L["layer"]] = {"Y": Y.clone()}
    ev[1].record()
    for L in reversed(layers):
        _, W, dY = pool[(L["shape"], L["pool"])]
        dX, dW = buf("dX", (n, L["d_in"])), buf("dW", (L["d_out"], L["d_in"]))
        rmm.rmm_backward(dY, W, xproj[L["layer"]], rmm.GAUSSIAN, L["seed"], L["offset"], dX=dX, dW=dW, ws=ws)
        if L["layer"] in keep:
            kept[L["layer"]].update(dX=dX.clone(), dW=dW.clone())
    ev[2].record()
    torch.cuda.synchronize()
    return xproj, kept, (ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]))


def test_config5_stack():
    S = synth.STACK
    layers = synth.stack_layers()
    assert len(layers) == 144 and S["k"] == synth.sketch_size(0.1, S["n"])
    host_pool = {(shape, p): synth.stack_pool_inputs(shape, p) for shape in ("attn", "ffn_up", "ffn_down") for p in range(3)}
    pool = {key: tuple(t.to(DEV) for t in v) for key, v in host_pool.items()}
    # first, middle and last block; of each: the first attention projection and the two FFN layers
    keep = {6 * blk + j for blk in (0, 12, 23) for j in (0, 4, 5)}

    xproj, kept, ms = run_stack(layers, pool, keep)
    print("stack forward %.2f ms, backward %.2f ms" % ms, flush=True)

    # stored activations: exactly k/n of X plus 16 bytes of state per layer
    saved = sum(x.numel() * x.element_size() + 16 for x in xproj)
    plain = sum(S["n"] * L["d_in"] * 2 for L in layers)
    o_saved = sum(o_rmm.saved_bytes(S["n"], L["d_in"], S["k"], 2)[0] for L in layers)
    assert saved == o_saved == 24 * (4 * 1024 + 1024 + 4096) * S["k"] * 2 + 144 * 16
    assert plain == 24 * (4 * 1024 + 1024 + 4096) * S["n"] * 2
    assert abs(saved / 1e9 - 0.7246) < 1e-4 and abs(plain / 1e9 - 7.2478) < 1e-4
    assert (saved - 144 * 16) * S["n"] == plain * S["k"]
    for x in xproj:
        assert bool(torch.isfinite(x.float()).all())

    # parity on the sampled layers
    for L in layers:
        if L["layer"] not in keep:
            continue
        X, W, dY = (synth.to_f64(t) for t in host_pool[(L["shape"], L["pool"])])
        oY, oXp = o_rmm.forward(X, W, None, S["k"], rmm.GAUSSIAN, L["seed"], L["offset"])
        odX, odW, _ = o_rmm.backward(dY, W, synth.to_f64(xproj[L["layer"]]), rmm.GAUSSIAN, L["seed"], L["offset"])
        _, odW_chain, _ = o_rmm.backward(dY, W, oXp, rmm.GAUSSIAN, L["seed"], L["offset"])
        got = kept[L["layer"]]
        errs = {"Y": rel_fro(got["Y"], oY), "X_proj": rel_fro(xproj[L["layer"]], oXp), "dX": rel_fro(got["dX"], odX),
                "dW": rel_fro(got["dW"], odW), "dW_chain": rel_fro(got["dW"], odW_chain)}
        print("layer %3d %-8s" % (L["layer"], L["shape"]), {k_: "%.2e" % v for k_, v in errs.items()}, flush=True)
        for name, e in errs.items():
            assert e <= 1e-2, (L["layer"], name, e)
        for name, g_, w_ in (("Y", got["Y"], oY), ("X_proj", xproj[L["layer"]], oXp), ("dX", got["dX"], odX),
                             ("dW", got["dW"], odW)):
            assert_close(g_, w_, name, "bf16", "stack layer %d" % L["layer"])

    # layers that share inputs but not the sketch state must differ; a second run must not
    assert not torch.equal(xproj[0], xproj[1])
    xproj2, kept2, _ = run_stack(layers, pool, keep)
    for a, b in zip(xproj, xproj2):
        assert torch.equal(a, b)
    for l in keep:
        for name in ("Y", "dX", "dW"):
            assert torch.equal(kept[l][name], kept2[l][name])
