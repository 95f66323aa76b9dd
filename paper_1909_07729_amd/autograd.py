"""``torch.autograd`` functions over the library's forward and gradient entry points, for training
through K-TanH as in Section 3 of arXiv:1909.07729 (the network is trained with K-TanH in place of
TanH and Sigmoid).

Plumbing only: each ``forward`` is one call of a forward entry point, each ``backward`` one call of
the matching gradient entry point; all arithmetic runs in the library's kernels.  Tensors are
``torch.bfloat16`` or ``torch.float32`` (the LSTM cell takes BFloat16 gates and a Float32 state),
on the GPU.  The gradient is the derivative identity of the exact function evaluated on the K-TanH output (``dy * (1 - y^2)``,
``dy * s * (1 - s)``, and the derivatives of the Swish and GELU identities); the tables get no
gradient.
"""
from __future__ import annotations

import torch

from . import binding


def _is_f32(x: torch.Tensor) -> bool:
    if x.dtype == torch.float32:
        return True
    if x.dtype == torch.bfloat16:
        return False
    raise TypeError(f"expected a bfloat16 or float32 tensor, got {x.dtype}")


class _FromOutput(torch.autograd.Function):
    """TanH and Sigmoid: the backward needs only the forward output."""

    @staticmethod
    def forward(ctx, x, lut, names):
        fwd_name, bwd_name = names[_is_f32(x)]
        y = getattr(binding, fwd_name)(x.contiguous(), lut=lut)
        ctx.save_for_backward(y)
        ctx.bwd_name = bwd_name
        return y

    @staticmethod
    def backward(ctx, dy):
        (y,) = ctx.saved_tensors
        return getattr(binding, ctx.bwd_name)(dy.contiguous(), y), None, None


class _FromInput(torch.autograd.Function):
    """Swish and GELU: the backward rebuilds the K-TanH value from the forward input."""

    @staticmethod
    def forward(ctx, x, lut, names):
        fwd_name, bwd_name = names[_is_f32(x)]
        x = x.contiguous()
        ctx.save_for_backward(x)
        ctx.lut, ctx.bwd_name = lut, bwd_name
        return getattr(binding, fwd_name)(x, lut=lut)

    @staticmethod
    def backward(ctx, dy):
        (x,) = ctx.saved_tensors
        return getattr(binding, ctx.bwd_name)(dy.contiguous(), x, lut=ctx.lut), None, None


# (forward entry point, gradient entry point) for BFloat16 [False] and Float32 [True] tensors
_TANH = {False: ("ktanh_bf16", "ktanh_bf16_backward"), True: ("ktanh_f32", "ktanh_f32_backward")}
_SIGMOID = {False: ("ksigmoid", "ksigmoid_backward"), True: ("ksigmoid_f32", "ksigmoid_f32_backward")}
_SWISH = {False: ("kswish", "kswish_backward"), True: ("kswish_f32", "kswish_f32_backward")}
_GELU = {False: ("kgelu", "kgelu_backward"), True: ("kgelu_f32", "kgelu_f32_backward")}


class _KLstmCell(torch.autograd.Function):
    @staticmethod
    def forward(ctx, gates, c_prev, lut):
        gates, c_prev = gates.contiguous(), c_prev.contiguous()
        c_next, h = binding.klstm_cell(gates.unsqueeze(0), c_prev, lut=lut)
        ctx.save_for_backward(gates, c_prev)
        ctx.lut = lut
        return h[0], c_next

    @staticmethod
    def backward(ctx, dh, dc_next):
        gates, c_prev = ctx.saved_tensors
        # an output that took no part in the loss arrives as None
        if dh is None:
            dh = torch.zeros((c_prev.shape[0], c_prev.shape[1]), dtype=gates.dtype, device=gates.device)
        if dc_next is None:
            dc_next = torch.zeros_like(c_prev)
        dgates, dc_prev = binding.klstm_cell_backward(gates, c_prev, dh.contiguous(),
                                                      dc_next.contiguous(), lut=ctx.lut)
        return dgates, dc_prev, None


def ktanh(x: torch.Tensor, lut=None) -> torch.Tensor:
    """K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromOutput.apply(x, lut, _TANH)


def ksigmoid(x: torch.Tensor, lut=None) -> torch.Tensor:
    """Sigmoid through K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromOutput.apply(x, lut, _SIGMOID)


def kswish(x: torch.Tensor, lut=None) -> torch.Tensor:
    """Swish through K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromInput.apply(x, lut, _SWISH)


def kgelu(x: torch.Tensor, lut=None) -> torch.Tensor:
    """GELU (tanh form) through K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromInput.apply(x, lut, _GELU)


def klstm_cell(gates: torch.Tensor, c_prev: torch.Tensor, lut=None):
    """One LSTM-cell step: gates [B, 4H] BFloat16 (i|f|g|o), c_prev [B, H] Float32.
    Returns (h [B, H] BFloat16, c [B, H] Float32), differentiable with respect to both inputs."""
    return _KLstmCell.apply(gates, c_prev, lut)
