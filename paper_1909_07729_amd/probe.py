"""Python front-end of ``libktanh_probe.so`` (``include/ktanh_probe.h``): the measurement yardsticks
the benchmark puts next to the K-TanH figures.  Marshalling only; not part of the product path."""
from __future__ import annotations

import ctypes
import os

import torch

from .binding import KtanhError, _BF16_VIEWS, _check, _stream_handle

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libktanh_probe.so")
SIGNATURES = {"ktanh_probe_copy": "ppns", "ktanh_probe_read": "ppns", "ktanh_probe_write": "pns",
              "ktanh_probe_read_wide": "ppns", "ktanh_probe_write_wide": "pns",
              "ktanh_probe_lstm": "ppppnnns"}
EXPORTS = tuple(SIGNATURES)

_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(LIB_PATH)
        kinds = {"p": ctypes.c_void_p, "n": ctypes.c_size_t, "s": ctypes.c_void_p}
        for name, params in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.argtypes = [kinds[k] for k in params]
            fn.restype = ctypes.c_int
        _lib = lib
    return _lib


def ktanh_probe_copy(x, out, stream=None):
    """Copies a 16-bit tensor with the launch of ``ktanh_bf16`` and no arithmetic."""
    _check(x, _BF16_VIEWS, "in")
    _check(out, _BF16_VIEWS, "out")
    if out.numel() != x.numel():
        raise ValueError("in and out differ in size")
    st = load_library().ktanh_probe_copy(x.data_ptr(), out.data_ptr(), x.numel(), _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, "ktanh_probe_copy")
    return out


def ktanh_probe_read(x: torch.Tensor, sink: torch.Tensor, stream=None, wide=False):
    """The loads of that launch alone over the bytes of ``x``; ``sink`` is 1 KiB of device scratch.
    ``wide``: 512-thread blocks instead of the library's 64."""
    if not (x.is_cuda and sink.is_cuda and x.is_contiguous() and sink.is_contiguous()):
        raise ValueError("x and sink must be contiguous CUDA tensors")
    if sink.numel() * sink.element_size() < 1024:
        raise ValueError("sink must hold 1 KiB")
    name = "ktanh_probe_read_wide" if wide else "ktanh_probe_read"
    st = getattr(load_library(), name)(x.data_ptr(), sink.data_ptr(), x.numel() * x.element_size(),
                                       _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)


def ktanh_probe_write(out: torch.Tensor, stream=None, wide=False):
    """The stores of that launch alone over the bytes of ``out``.  ``wide``: 512-thread blocks."""
    if not (out.is_cuda and out.is_contiguous()):
        raise ValueError("out must be a contiguous CUDA tensor")
    name = "ktanh_probe_write_wide" if wide else "ktanh_probe_write"
    st = getattr(load_library(), name)(out.data_ptr(), out.numel() * out.element_size(), _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)


def ktanh_probe_lstm(gates: torch.Tensor, c_in: torch.Tensor, c_out: torch.Tensor, h_out: torch.Tensor,
                     stream=None):
    """The launch of ``klstm_cell`` with the arithmetic taken out: gates [T, B, 4H] 16-bit, c [B, H]
    Float32, h_out [T, B, H] 16-bit."""
    _check(gates, _BF16_VIEWS, "gates")
    _check(h_out, _BF16_VIEWS, "h_out")
    T, B, H4 = gates.shape
    H = H4 // 4
    if tuple(h_out.shape) != (T, B, H) or tuple(c_in.shape) != (B, H) or tuple(c_out.shape) != (B, H):
        raise ValueError("shapes: gates [T, B, 4H], c_in and c_out [B, H], h_out [T, B, H]")
    for name, t in (("c_in", c_in), ("c_out", c_out)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32):
            raise ValueError(f"{name} must be a contiguous CUDA Float32 tensor")
    st = load_library().ktanh_probe_lstm(gates.data_ptr(), c_in.data_ptr(), c_out.data_ptr(),
                                         h_out.data_ptr(), T, B, H, _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, "ktanh_probe_lstm")
    return h_out
