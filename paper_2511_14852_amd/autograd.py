"""torch.autograd access to the library: a Chebyshev-KAN stack as one differentiable function.

Argument marshalling and buffer allocation only: forward and backward of every layer run in the
HIP library (chebykan_stack_forward / chebykan_stack_backward); nothing here computes.  Layers are
chained directly (the output of one layer is the input of the next), as the paper's three-layer
stacks are (Sec. 6.1, Table 2); the backward pass regenerates the basis from the saved layer
inputs, nothing else is kept from forward.
"""
from __future__ import annotations

import torch

from . import binding


class ChebyKANStackFunction(torch.autograd.Function):
    """y = stack(x; C_0, ..., C_{n-1});  C_l has shape [in_l, out_l, degree+1]."""

    @staticmethod
    def forward(ctx, x, *Cs):
        x = x.contiguous()
        Cs = [c.contiguous() for c in Cs]
        B = x.shape[0]
        acts = [x] + [torch.empty((B, c.shape[1]), dtype=torch.float32, device=x.device) for c in Cs]
        widths = [int(Cs[0].shape[0])] + [int(c.shape[1]) for c in Cs]
        ws = binding.alloc_stack_workspace(B, widths, int(Cs[0].shape[2]) - 1, x.device)
        binding.chebykan_stack_forward(Cs, acts, ws)
        ctx.save_for_backward(*acts[:-1], *Cs)
        ctx.n_layers = len(Cs)
        return acts[-1]

    @staticmethod
    def backward(ctx, dy):
        n = ctx.n_layers
        saved = ctx.saved_tensors
        acts, Cs = list(saved[:n]), list(saved[n:])
        B = acts[0].shape[0]
        need_dx = ctx.needs_input_grad[0]
        grads = [torch.empty_like(a) if (l > 0 or need_dx) else None for l, a in enumerate(acts)] + [dy.contiguous()]
        dCs = [torch.empty_like(c) if ctx.needs_input_grad[1 + l] else None for l, c in enumerate(Cs)]
        if grads[0] is None and dCs[0] is None:      # the first layer needs at least one output
            dCs[0] = torch.empty_like(Cs[0])
        widths = [int(Cs[0].shape[0])] + [int(c.shape[1]) for c in Cs]
        ws = binding.alloc_stack_workspace(B, widths, int(Cs[0].shape[2]) - 1, dy.device)
        binding.chebykan_stack_backward(Cs, acts, grads, dCs, ws)
        return (grads[0] if need_dx else None, *[d if ctx.needs_input_grad[1 + l] else None for l, d in enumerate(dCs)])


class ChebyKANStack(torch.nn.Module):
    """A stack of Chebyshev-KAN layers of one degree; coefficients ~ N(0, 1/(in*(degree+1)))."""

    def __init__(self, widths, degree: int, device="cuda"):
        super().__init__()
        self.widths, self.degree = [int(w) for w in widths], int(degree)
        self.coeffs = torch.nn.ParameterList()
        for i, o in zip(self.widths[:-1], self.widths[1:]):
            std = 1.0 / (i * (degree + 1)) ** 0.5
            self.coeffs.append(torch.nn.Parameter(torch.randn(i, o, degree + 1, device=device) * std))

    def forward(self, x):
        return ChebyKANStackFunction.apply(x, *self.coeffs)
