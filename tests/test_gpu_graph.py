"""GPU: a forward + backward pass captured in a HIP graph (the library allocates nothing, never
synchronises and records no memset, so its calls can be captured) replays to the eager result,
several times, with eager work and synchronisations between the replays."""
import pytest
import torch

import paper_2201_13195_amd as rmm
from paper_2201_13195_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("kind", [rmm.GAUSSIAN, rmm.RADEMACHER])
def test_captured_step_replays_to_the_eager_result(kind):
    n, d_in, d_out, k = 2048, 512, 1024, 205
    X, W, dY = (t.to(DEV) for t in synth.layer_inputs(n, d_in, d_out, "bf16", (95, 96, 97)))
    bias = synth.to_torch(synth.normal((d_out,), 98), "bf16").to(DEV)
    ws = torch.empty(max(rmm.rmm_workspace_bytes(n, d_in, d_out, k, torch.bfloat16, kind, op) for op in (0, 1)) + 16,
                     dtype=torch.uint8, device=DEV)
    out = dict(Y=torch.empty((n, d_out), dtype=torch.bfloat16, device=DEV),
               Xp=torch.empty((k, d_in), dtype=torch.bfloat16, device=DEV),
               dX=torch.empty((n, d_in), dtype=torch.bfloat16, device=DEV),
               dW=torch.empty((d_out, d_in), dtype=torch.bfloat16, device=DEV),
               db=torch.empty((d_out,), dtype=torch.bfloat16, device=DEV))

    def step():
        rmm.rmm_forward(X, W, bias, k, kind, 11, 5, Y=out["Y"], X_proj=out["Xp"], ws=ws)
        rmm.rmm_backward(dY, W, out["Xp"], kind, 11, 5, need_dbias=True, dX=out["dX"], dW=out["dW"], dbias=out["db"],
                         ws=ws)

    step()
    torch.cuda.synchronize()
    eager = {name: t.clone() for name, t in out.items()}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(4):
        for t in out.values():
            t.zero_()                            # eager work between the replays
        ws.fill_(replay + 1)                     # the workspace content must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t in out.items():
            assert torch.equal(t, eager[name]), (replay, name)
