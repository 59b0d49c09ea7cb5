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


class _Projection(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, Wx, bias, n_heads):
        ctx.n_heads = n_heads
        ctx.has_bias = bias is not None
        ctx.save_for_backward(x, Wx)
        return binding.input_projection(x, Wx, bias, n_heads=n_heads)

    @staticmethod
    def backward(ctx, du):
        x, Wx = ctx.saved_tensors
        need_x, need_w, need_b = ctx.needs_input_grad[0], ctx.needs_input_grad[1], ctx.has_bias and ctx.needs_input_grad[2]
        dx, dW, db = binding.input_projection_backward(x, Wx, du.contiguous(), n_heads=ctx.n_heads, want_dx=need_x,
                                                       want_dw=need_w or need_b, want_dbias=need_b)
        return dx, (dW if need_w else None), db, None


def input_projection_apply(x, Wx, bias=None, n_heads: int = 1):
    """u = B x + b for all gates (multi-head input matrices), differentiable with respect to x, Wx
    and bias: pararnn_input_projection with pararnn_input_projection_backward as its gradient."""
    return _Projection.apply(x, Wx, bias, n_heads)


def rnn_layer(cell, x, Wx, bias, params, h0=None, n_heads: int = 1, tol: float = 1e-6, max_iter: int = 64):
    """The paper's cell applied to a sequence: the input projection followed by the Newton solve of
    the recurrence, differentiable end to end.  Returns (h, iters)."""
    return rnn_apply(cell, params, input_projection_apply(x, Wx, bias, n_heads), h0, tol, max_iter)


def rnn_apply(cell: str, params, u, h0=None, tol: float = 1e-6, max_iter: int = 64):
    """h = RNN(u) by the Newton solve, differentiable with respect to params, u
    and h0 (Eq. (6)).  Returns (h, iters); iters is the device int32[2] tensor
    {iterations, status} of pararnn_forward."""
    return _ParaRNN.apply(params, u, h0, cell, tol, max_iter)
