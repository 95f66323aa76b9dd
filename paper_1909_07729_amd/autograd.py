"""``torch.autograd`` functions over the library's forward and gradient entry points, for training
through K-TanH as in Section 3 of arXiv:1909.07729 (the network is trained with K-TanH in place of
TanH and Sigmoid).

Plumbing only: each ``forward`` is one call of a forward entry point, each ``backward`` one call of
the matching gradient entry point; all arithmetic runs in the library's kernels.  Tensors are
``torch.bfloat16`` or ``torch.float32`` (the LSTM cell takes BFloat16 gates and a Float32 state),
on the GPU.  The gradient is the derivative identity of the exact function evaluated on the K-TanH output (``dy * (1 - y^2)``,
``dy * s * (1 - s)``, and the derivatives of the Swish and GELU identities); the tables get no
gradient.  Every function takes ``lut`` (a ``KtanhLut`` or a ``KtanhLut64``; None = the default
table) and ``intervals`` (32 or 64: which default table and which entry points; a ``KtanhLut64``
selects 64 by itself).
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


def _is_wide(lut, intervals: int) -> bool:
    if isinstance(lut, binding.KtanhLut64):
        return True
    if intervals not in (32, 64):
        raise ValueError("intervals must be 32 or 64")
    if lut is not None and intervals == 64:
        raise TypeError("intervals=64 needs a KtanhLut64 (or lut=None for the fitted table)")
    return intervals == 64


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


# (forward entry point, gradient entry point) by table width [wide] and tensor type [Float32];
# the gradients of TanH and Sigmoid read the forward output and no table, so they serve both widths
_TANH = {False: {False: ("ktanh_bf16", "ktanh_bf16_backward"), True: ("ktanh_f32", "ktanh_f32_backward")},
         True: {False: ("ktanh64_bf16", "ktanh_bf16_backward"), True: ("ktanh64_f32", "ktanh_f32_backward")}}
_SIGMOID = {False: {False: ("ksigmoid", "ksigmoid_backward"), True: ("ksigmoid_f32", "ksigmoid_f32_backward")},
            True: {False: ("ksigmoid64", "ksigmoid_backward"), True: ("ksigmoid64_f32", "ksigmoid_f32_backward")}}
_SWISH = {False: {False: ("kswish", "kswish_backward"), True: ("kswish_f32", "kswish_f32_backward")},
          True: {False: ("kswish64", "kswish64_backward"), True: ("kswish64_f32", "kswish64_f32_backward")}}
_GELU = {False: {False: ("kgelu", "kgelu_backward"), True: ("kgelu_f32", "kgelu_f32_backward")},
         True: {False: ("kgelu64", "kgelu64_backward"), True: ("kgelu64_f32", "kgelu64_f32_backward")}}


class _KLstmCell(torch.autograd.Function):
    @staticmethod
    def forward(ctx, gates, c_prev, lut, wide):
        gates, c_prev = gates.contiguous(), c_prev.contiguous()
        cell = binding.klstm_cell64 if wide else binding.klstm_cell
        c_next, h = cell(gates.unsqueeze(0), c_prev, lut=lut)
        ctx.save_for_backward(gates, c_prev)
        ctx.lut, ctx.wide = lut, wide
        return h[0], c_next

    @staticmethod
    def backward(ctx, dh, dc_next):
        gates, c_prev = ctx.saved_tensors
        # an output that took no part in the loss arrives as None
        if dh is None:
            dh = torch.zeros((c_prev.shape[0], c_prev.shape[1]), dtype=gates.dtype, device=gates.device)
        if dc_next is None:
            dc_next = torch.zeros_like(c_prev)
        cell_backward = binding.klstm_cell64_backward if ctx.wide else binding.klstm_cell_backward
        dgates, dc_prev = cell_backward(gates, c_prev, dh.contiguous(), dc_next.contiguous(), lut=ctx.lut)
        return dgates, dc_prev, None, None


def ktanh(x: torch.Tensor, lut=None, intervals: int = 32) -> torch.Tensor:
    """K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromOutput.apply(x, lut, _TANH[_is_wide(lut, intervals)])


def ksigmoid(x: torch.Tensor, lut=None, intervals: int = 32) -> torch.Tensor:
    """Sigmoid through K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromOutput.apply(x, lut, _SIGMOID[_is_wide(lut, intervals)])


def kswish(x: torch.Tensor, lut=None, intervals: int = 32) -> torch.Tensor:
    """Swish through K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromInput.apply(x, lut, _SWISH[_is_wide(lut, intervals)])


def kgelu(x: torch.Tensor, lut=None, intervals: int = 32) -> torch.Tensor:
    """GELU (tanh form) through K-TanH of a BFloat16 or Float32 tensor, differentiable with respect to ``x``."""
    return _FromInput.apply(x, lut, _GELU[_is_wide(lut, intervals)])


def klstm_cell(gates: torch.Tensor, c_prev: torch.Tensor, lut=None, intervals: int = 32):
    """One LSTM-cell step: gates [B, 4H] BFloat16 (i|f|g|o), c_prev [B, H] Float32.
    Returns (h [B, H] BFloat16, c [B, H] Float32), differentiable with respect to both inputs."""
    return _KLstmCell.apply(gates, c_prev, lut, _is_wide(lut, intervals))
