"""``torch.autograd`` functions over the library's forward and gradient entry points, for training
through K-TanH as in Section 3 of arXiv:1909.07729 (the network is trained with K-TanH in place of
TanH and Sigmoid).

Plumbing only: each ``forward`` is one call of a forward entry point, each ``backward`` one call of
the matching gradient entry point; all arithmetic runs in the library's kernels.  Tensors are
``torch.bfloat16`` (Float32 for the LSTM cell state), on the GPU.  The gradient is the derivative
identity of the exact function evaluated on the K-TanH output (``dy * (1 - y^2)``,
``dy * s * (1 - s)``, and the derivatives of the Swish and GELU identities); the tables get no
gradient.
"""
from __future__ import annotations

import torch

from . import binding


class _KTanh(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, lut):
        y = binding.ktanh_bf16(x.contiguous(), lut=lut)
        ctx.save_for_backward(y)
        return y

    @staticmethod
    def backward(ctx, dy):
        (y,) = ctx.saved_tensors
        return binding.ktanh_bf16_backward(dy.contiguous(), y), None


class _KSigmoid(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, lut):
        s = binding.ksigmoid(x.contiguous(), lut=lut)
        ctx.save_for_backward(s)
        return s

    @staticmethod
    def backward(ctx, dy):
        (s,) = ctx.saved_tensors
        return binding.ksigmoid_backward(dy.contiguous(), s), None


class _KSwish(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, lut):
        x = x.contiguous()
        ctx.save_for_backward(x)
        ctx.lut = lut
        return binding.kswish(x, lut=lut)

    @staticmethod
    def backward(ctx, dy):
        (x,) = ctx.saved_tensors
        return binding.kswish_backward(dy.contiguous(), x, lut=ctx.lut), None


class _KGelu(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, lut):
        x = x.contiguous()
        ctx.save_for_backward(x)
        ctx.lut = lut
        return binding.kgelu(x, lut=lut)

    @staticmethod
    def backward(ctx, dy):
        (x,) = ctx.saved_tensors
        return binding.kgelu_backward(dy.contiguous(), x, lut=ctx.lut), None


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
    """K-TanH of a BFloat16 tensor, differentiable with respect to ``x``."""
    return _KTanh.apply(x, lut)


def ksigmoid(x: torch.Tensor, lut=None) -> torch.Tensor:
    """Sigmoid through K-TanH of a BFloat16 tensor, differentiable with respect to ``x``."""
    return _KSigmoid.apply(x, lut)


def kswish(x: torch.Tensor, lut=None) -> torch.Tensor:
    """Swish through K-TanH of a BFloat16 tensor, differentiable with respect to ``x``."""
    return _KSwish.apply(x, lut)


def kgelu(x: torch.Tensor, lut=None) -> torch.Tensor:
    """GELU (tanh form) through K-TanH of a BFloat16 tensor, differentiable with respect to ``x``."""
    return _KGelu.apply(x, lut)


def klstm_cell(gates: torch.Tensor, c_prev: torch.Tensor, lut=None):
    """One LSTM-cell step: gates [B, 4H] BFloat16 (i|f|g|o), c_prev [B, H] Float32.
    Returns (h [B, H] BFloat16, c [B, H] Float32), differentiable with respect to both inputs."""
    return _KLstmCell.apply(gates, c_prev, lut)
