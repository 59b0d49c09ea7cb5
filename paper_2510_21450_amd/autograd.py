"""torch.autograd glue over the binding: `rnn_apply` runs pararnn_forward and
registers pararnn_backward as its gradient, so the library can sit inside a
PyTorch training step.  No arithmetic happens here: both directions run in the
HIP kernels, on the current stream."""
import torch

from . import binding


class _ParaRNN(torch.autograd.Function):
    @staticmethod
    def forward(ctx, params, u, h0, cell, tol, max_iter):
        h, iters, _ = binding.forward(cell, params, u, h0, tol=tol, max_iter=max_iter)
        ctx.cell = cell
        ctx.save_for_backward(params, u, h0 if h0 is not None else torch.empty(0, device=u.device), h)
        ctx.has_h0 = h0 is not None
        ctx.mark_non_differentiable(iters)
        return h, iters

    @staticmethod
    def backward(ctx, dL_dh, _unused):
        params, u, h0, h = ctx.saved_tensors
        h0 = h0 if ctx.has_h0 else None
        want_dh0 = ctx.has_h0 and ctx.needs_input_grad[2]
        du, dparams, dh0 = binding.backward(ctx.cell, params, u, h0, h, dL_dh.contiguous(), want_dh0=want_dh0)
        return dparams, du, dh0, None, None, None


def rnn_apply(cell: str, params, u, h0=None, tol: float = 1e-6, max_iter: int = 64):
    """h = RNN(u) by the Newton solve, differentiable with respect to params, u
    and h0 (Eq. (6)).  Returns (h, iters); iters is the device int32[2] tensor
    {iterations, status} of pararnn_forward."""
    return _ParaRNN.apply(params, u, h0, cell, tol, max_iter)
