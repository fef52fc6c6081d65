"""Drop-in layer over the C ABI: `torch.autograd.Function` + `nn.Module` form of Algorithm 1
(the paper's user-facing form, Section 3: a linear layer whose backward uses the sketched input).

Argument marshalling only: the forward is one `rmm_forward` call, the backward one
`rmm_backward` call; autograd keeps X_proj and the 16-byte sketch state, not X (Section 2.4.1).
"""
import itertools

import torch

from . import binding

_layer_ids = itertools.count()     # process-wide: layers built without an explicit layer_id get distinct ones


class RMMLinearFunction(torch.autograd.Function):
    """Y = X W^T (+ b); backward: dX = dY W exactly, dW = (S^T dY)^T (S^T X), db = dY^T 1."""

    @staticmethod
    def forward(ctx, X, W, bias, k, kind, seed, offset):
        lead = X.shape[:-1]
        X2 = X.reshape(-1, X.shape[-1])
        if not X2.is_contiguous():
            X2 = X2.contiguous()
        Wc = W if W.is_contiguous() else W.contiguous()
        Y, X_proj = binding.rmm_forward(X2, Wc, bias, k, kind, seed, offset)
        ctx.save_for_backward(Wc, X_proj)          # X itself is not kept
        ctx.state = (kind, seed, offset)
        ctx.lead, ctx.has_bias = lead, bias is not None
        return Y.reshape(*lead, W.shape[0])

    @staticmethod
    def backward(ctx, dY):
        W, X_proj = ctx.saved_tensors
        kind, seed, offset = ctx.state
        dY2 = dY.reshape(-1, dY.shape[-1])
        if not dY2.is_contiguous():
            dY2 = dY2.contiguous()
        dX, dW, db = binding.rmm_backward(dY2, W, X_proj, kind, seed, offset, need_dX=ctx.needs_input_grad[0],
                                          need_dbias=ctx.has_bias and ctx.needs_input_grad[2])
        if dX is not None:
            dX = dX.reshape(*ctx.lead, W.shape[1])
        return dX, dW, db, None, None, None, None


class RMMLinear(torch.nn.Module):
    """`nn.Linear` replacement.  The sketch size is `k` tokens, or `round(rho * n)` of the n
    tokens of each call (clamped to [1, n]); every forward call that will be followed by a
    backward call draws a fresh sketch: state (seed, offset = layer_id * 2^32 + call counter), so
    that sketches of different layers and steps are independent of each other and of dY
    (Section 2.1).  `layer_id` defaults to a process-wide running number.  With gradients disabled
    the layer computes Y only: no sketch, no state consumed."""

    def __init__(self, in_features, out_features, bias=True, rho=0.1, k=None, kind=binding.GAUSSIAN, seed=0,
                 layer_id=None, device="cuda", dtype=torch.bfloat16):
        super().__init__()
        self.in_features, self.out_features = in_features, out_features
        self.rho, self.k, self.kind, self.seed = rho, k, kind, seed
        self.layer_id = next(_layer_ids) if layer_id is None else int(layer_id)
        self.calls = 0
        self.weight = torch.nn.Parameter(torch.empty((out_features, in_features), device=device, dtype=dtype))
        self.bias = torch.nn.Parameter(torch.zeros((out_features,), device=device, dtype=dtype)) if bias else None
        torch.nn.init.normal_(self.weight, std=0.02)

    def sketch_size(self, n):
        k = self.k if self.k is not None else int(self.rho * n + 0.5)
        return max(1, min(int(k), n))

    def next_state(self):
        offset = (self.layer_id << 32) | (self.calls & 0xFFFFFFFF)
        self.calls += 1
        return self.seed, offset

    def forward(self, X):
        n = X.numel() // X.shape[-1]
        if not torch.is_grad_enabled():        # nothing will be kept for a backward pass: Y alone
            X2 = X.reshape(-1, X.shape[-1]).contiguous()
            Y, _ = binding.rmm_forward(X2, self.weight.detach().contiguous(), self.bias, 1, self.kind, 0, 0,
                                       need_xproj=False)
            return Y.reshape(*X.shape[:-1], self.out_features)
        seed, offset = self.next_state()
        self.last_state = (seed, offset)
        return RMMLinearFunction.apply(X, self.weight, self.bias, self.sketch_size(n), self.kind, seed, offset)
