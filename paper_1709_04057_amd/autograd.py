"""torch.autograd wrappers around the liblinrec entry points.

Each function here only wires a forward entry point to its backward entry point so that PyTorch's
autograd can differentiate through the recurrence; all arithmetic stays in the library's HIP kernels
(arXiv 1709.04057: Section 2.2 gives the backward pass of the plain recurrence, the gated forms of
Sections 3.1 and 3.2 follow by the chain rule inside the kernels).  Tensors are time-major
``[T, B, n]`` float32 on the GPU; the initial state is ``[B, n]`` or None.
"""
from __future__ import annotations

import torch

from . import binding as _b


def _c(t):
    return None if t is None else t.contiguous()


class _LinearRecurrence(torch.autograd.Function):
    @staticmethod
    def forward(ctx, lam, x, h0):
        lam, x, h0 = _c(lam), _c(x), _c(h0)
        h = _b.linrec_forward(lam, x, h0)
        ctx.save_for_backward(lam, h, h0 if h0 is not None else lam.new_empty(0))
        ctx.has_h0 = h0 is not None
        return h

    @staticmethod
    def backward(ctx, grad_h):
        lam, h, h0 = ctx.saved_tensors
        h0 = h0 if ctx.has_h0 else None
        need = ctx.needs_input_grad
        gx, gl, gh0 = _b.linrec_backward(lam, h, h0, _c(grad_h), want_grad_x=need[1], want_grad_lambda=need[0],
                                         want_grad_h0=need[2] and ctx.has_h0)
        return gl, gx, gh0


def linear_recurrence(lam, x, h0=None):
    """``h[t] = lam[t] * h[t-1] + x[t]`` with ``h[-1] = h0`` (zeros when None); differentiable in all three."""
    return _LinearRecurrence.apply(lam, x, h0)


class _Gilr(torch.autograd.Function):
    @staticmethod
    def forward(ctx, g_pre, i_pre, h0, tau):
        g_pre, i_pre, h0 = _c(g_pre), _c(i_pre), _c(h0)
        h = _b.linrec_gilr_forward(g_pre, i_pre, h0, tau=tau)
        ctx.save_for_backward(g_pre, i_pre, h, h0 if h0 is not None else g_pre.new_empty(0))
        ctx.has_h0, ctx.tau = h0 is not None, tau
        return h

    @staticmethod
    def backward(ctx, grad_h):
        g_pre, i_pre, h, h0 = ctx.saved_tensors
        h0 = h0 if ctx.has_h0 else None
        need = ctx.needs_input_grad
        gg, gi, gh0 = _b.linrec_gilr_backward(g_pre, i_pre, h, h0, _c(grad_h), tau=ctx.tau, want_grad_g_pre=need[0],
                                              want_grad_i_pre=need[1], want_grad_h0=need[2] and ctx.has_h0)
        return gg, gi, gh0, None


def gilr(g_pre, i_pre, h0=None, tau=_b.TAU_TANH):
    """Gated impulse linear recurrent layer after its matrix products:
    ``h[t] = g*h[t-1] + (1-g)*tau(i_pre[t])``, ``g = sigmoid(g_pre[t])``."""
    return _Gilr.apply(g_pre, i_pre, h0, int(tau))


class _LstmCell(torch.autograd.Function):
    @staticmethod
    def forward(ctx, f_pre, i_pre, z_pre, o_pre, c0):
        f_pre, i_pre, z_pre, o_pre, c0 = (_c(t) for t in (f_pre, i_pre, z_pre, o_pre, c0))
        c, h = _b.linrec_lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0)
        ctx.save_for_backward(f_pre, i_pre, z_pre, o_pre, c, c0 if c0 is not None else f_pre.new_empty(0))
        ctx.has_c0 = c0 is not None
        ctx.mark_non_differentiable(c)
        return h, c

    @staticmethod
    def backward(ctx, grad_h, _grad_c):
        f_pre, i_pre, z_pre, o_pre, c, c0 = ctx.saved_tensors
        c0 = c0 if ctx.has_c0 else None
        need = ctx.needs_input_grad
        gf, gi, gz, go, gc0 = _b.linrec_lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, _c(grad_h),
                                                           want=tuple(need[:4]), want_grad_c0=need[4] and ctx.has_c0)
        return gf, gi, gz, go, gc0


def lstm_cell(f_pre, i_pre, z_pre, o_pre, c0=None):
    """Cell of the GILR-LSTM: ``c[t] = f*c[t-1] + i*z``, ``h[t] = o*c[t]``; returns ``(h, c)``.

    Gradients flow through ``h`` only: ``c`` is returned for inspection and for carrying the state into
    the next segment, and is marked non-differentiable (the library's backward entry point takes dL/dh)."""
    return _LstmCell.apply(f_pre, i_pre, z_pre, o_pre, c0)
