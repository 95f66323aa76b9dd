"""Python front-end of the C-ABI library ``libktanh.so``: argument marshalling only.

Each function below has the name of the C entry point it calls (``include/ktanh.h``).  Tensors are
``torch`` CUDA tensors used purely as device memory; every step of the computation runs inside the
library's HIP kernels, on the current torch stream.  There is no fallback: if the library has not
been built, or a call is rejected, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libktanh.so")
INTERVALS = 32

# Every function include/ktanh.h declares, with the kinds of its parameters:
#   p = device tensor pointer, n = size_t, l = table pointer (32 intervals), L = table pointer (64),
#   s = stream, i = int status.  The ctypes prototypes below are built from these strings and nothing else.
SIGNATURES = {
    "ktanh_status_string": "i", "ktanh_default_lut": "", "ktanh_lut_validate": "l",
    "ktanh_lut64_validate": "L", "ktanh_fit_lut": "l", "ktanh_fit_lut64": "L", "ktanh_fit_lut_bmin0": "l",
    "ktanh_bf16": "ppnls", "ktanh_f32": "ppnls", "ksigmoid": "ppnls", "kswish": "ppnls", "kgelu": "ppnls",
    "ktanh64_bf16": "ppnLs", "ktanh64_f32": "ppnLs", "ksigmoid64": "ppnLs", "kswish64": "ppnLs",
    "kgelu64": "ppnLs",
    "ksigmoid_f32": "ppnls", "kswish_f32": "ppnls", "kgelu_f32": "ppnls", "ktanh_f32_to_bf16": "ppnls",
    "ksigmoid64_f32": "ppnLs", "kswish64_f32": "ppnLs", "kgelu64_f32": "ppnLs",
    "klstm_cell": "ppppnnnls", "klstm_cell64": "ppppnnnLs",
    "ktanh_bf16_backward": "pppns", "ksigmoid_backward": "pppns",
    "ktanh_f32_backward": "pppns", "ksigmoid_f32_backward": "pppns",
    "kswish_backward": "pppnls", "kgelu_backward": "pppnls",
    "kswish_f32_backward": "pppnls", "kgelu_f32_backward": "pppnls",
    "kswish64_backward": "pppnLs", "kgelu64_backward": "pppnLs",
    "kswish64_f32_backward": "pppnLs", "kgelu64_f32_backward": "pppnLs",
    "klstm_cell_backward": "ppppppnnls", "klstm_cell64_backward": "ppppppnnLs",
    "kpade32_bf16": "ppns", "kpade78_bf16": "ppns",
    "ktaylor2_bf16": "ppns", "ktaylor3_bf16": "ppns",
}
EXPORTS = tuple(SIGNATURES)


class KtanhLut(ctypes.Structure):
    """Mirror of ``ktanh_lut_t``: the tables T_E, T_r, T_b of Algorithm 1, indexed by t."""

    _fields_ = [
        ("E", ctypes.c_uint8 * INTERVALS),
        ("r", ctypes.c_uint8 * INTERVALS),
        ("b", ctypes.c_int8 * INTERVALS),
    ]

    @classmethod
    def from_tuples(cls, rows):
        lut = cls()
        for t, (E, r, b) in enumerate(rows):
            lut.E[t], lut.r[t], lut.b[t] = E, r, b
        return lut

    def as_tuples(self):
        return [(int(self.E[t]), int(self.r[t]), int(self.b[t])) for t in range(INTERVALS)]


class KtanhLut64(ctypes.Structure):
    """Mirror of ``ktanh_lut64_t``: 64-interval tables, t = (E_i & 3) << 4 | (M_i >> 3)."""

    _fields_ = [
        ("E", ctypes.c_uint8 * 64),
        ("r", ctypes.c_uint8 * 64),
        ("b", ctypes.c_int8 * 64),
    ]

    @classmethod
    def from_tuples(cls, rows):
        lut = cls()
        for t, (E, r, b) in enumerate(rows):
            lut.E[t], lut.r[t], lut.b[t] = E, r, b
        return lut

    def as_tuples(self):
        return [(int(self.E[t]), int(self.r[t]), int(self.b[t])) for t in range(64)]


class KtanhError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libktanh.so (once).  Raises if it is missing: build it with ``__graft_entry__.build()``."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(LIB_PATH)
        kinds = {"p": ctypes.c_void_p, "n": ctypes.c_size_t, "s": ctypes.c_void_p, "i": ctypes.c_int,
                 "l": ctypes.POINTER(KtanhLut), "L": ctypes.POINTER(KtanhLut64)}
        for name, params in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.argtypes = [kinds[k] for k in params]
            fn.restype = ctypes.c_int
        lib.ktanh_status_string.restype = ctypes.c_char_p
        lib.ktanh_default_lut.restype = ctypes.POINTER(KtanhLut)
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().ktanh_status_string(int(status)).decode()


def ktanh_default_lut() -> KtanhLut:
    """A copy of the library's built-in table (Table 1 of the paper)."""
    src = load_library().ktanh_default_lut().contents
    dst = KtanhLut()
    ctypes.memmove(ctypes.byref(dst), ctypes.byref(src), ctypes.sizeof(KtanhLut))
    return dst


def ktanh_lut_validate(lut: KtanhLut | None) -> int:
    return load_library().ktanh_lut_validate(ctypes.byref(lut) if lut is not None else None)


def ktanh_fit_lut() -> KtanhLut:
    """The 32-interval table from the library's own fit of Section 2.4 (equals Table 1)."""
    lut = KtanhLut()
    st = load_library().ktanh_fit_lut(ctypes.byref(lut))
    if st != 0:
        raise KtanhError(st, "ktanh_fit_lut")
    return lut


def ktanh_fit_lut_bmin0() -> KtanhLut:
    """The ablation's sub-optimal table: the fit of Section 2.4 with b_min = 0."""
    lut = KtanhLut()
    st = load_library().ktanh_fit_lut_bmin0(ctypes.byref(lut))
    if st != 0:
        raise KtanhError(st, "ktanh_fit_lut_bmin0")
    return lut


def ktanh_fit_lut64() -> KtanhLut64:
    """The 64-interval table from the library's fit."""
    lut = KtanhLut64()
    st = load_library().ktanh_fit_lut64(ctypes.byref(lut))
    if st != 0:
        raise KtanhError(st, "ktanh_fit_lut64")
    return lut


def ktanh_lut64_validate(lut: KtanhLut64 | None) -> int:
    return load_library().ktanh_lut64_validate(ctypes.byref(lut) if lut is not None else None)


def _stream_handle(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _lut_arg(lut):
    return None if lut is None else ctypes.byref(lut)


_BF16_VIEWS = (torch.bfloat16, torch.int16, torch.uint16)
_F32_VIEWS = (torch.float32, torch.int32, torch.uint32)


def _check(t: torch.Tensor, dtypes, what: str):
    if not t.is_cuda:
        raise ValueError(f"{what} must be a CUDA tensor (device memory)")
    if t.dtype not in dtypes:
        raise TypeError(f"{what} has dtype {t.dtype}, expected one of {dtypes}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")


def _elementwise(name, x, out, lut, stream, dtypes):
    _check(x, dtypes, "in")
    if out is None:
        out = torch.empty_like(x)
    _check(out, dtypes, "out")
    if out.numel() != x.numel():
        raise ValueError("in and out differ in size")
    st = getattr(load_library(), name)(x.data_ptr(), out.data_ptr(), x.numel(), _lut_arg(lut),
                                       _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)
    return out


def ktanh_bf16(x, out=None, lut=None, stream=None):
    """K-TanH on a BFloat16 tensor (or its int16/uint16 bit view); ``out`` may be ``x``."""
    return _elementwise("ktanh_bf16", x, out, lut, stream, _BF16_VIEWS)


def _pade(name, x, out, stream):
    _check(x, _BF16_VIEWS, "in")
    if out is None:
        out = torch.empty_like(x)
    _check(out, _BF16_VIEWS, "out")
    if out.numel() != x.numel():
        raise ValueError("in and out differ in size")
    st = getattr(load_library(), name)(x.data_ptr(), out.data_ptr(), x.numel(), _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)
    return out


def kpade32_bf16(x, out=None, stream=None):
    """The Pade[3/2] approximant of TanH (a comparison row of the paper's Table 2) on BFloat16."""
    return _pade("kpade32_bf16", x, out, stream)


def kpade78_bf16(x, out=None, stream=None):
    """The Pade[7/8] approximant of TanH (a comparison row of the paper's Table 2) on BFloat16."""
    return _pade("kpade78_bf16", x, out, stream)


def ktaylor2_bf16(x, out=None, stream=None):
    """Piecewise Taylor polynomials of degree 2 on K-TanH's intervals (a comparison row of Table 2)."""
    return _pade("ktaylor2_bf16", x, out, stream)


def ktaylor3_bf16(x, out=None, stream=None):
    """The same of degree 3."""
    return _pade("ktaylor3_bf16", x, out, stream)


def ktanh_f32(x, out=None, lut=None, stream=None):
    """K-TanH on a Float32 tensor (or its int32/uint32 bit view)."""
    return _elementwise("ktanh_f32", x, out, lut, stream, _F32_VIEWS)


def ktanh64_bf16(x, out=None, lut=None, stream=None):
    """K-TanH with a 64-interval table (``KtanhLut64``; None = the fitted one) on BFloat16."""
    return _elementwise("ktanh64_bf16", x, out, lut, stream, _BF16_VIEWS)


def ktanh64_f32(x, out=None, lut=None, stream=None):
    """K-TanH with a 64-interval table on Float32."""
    return _elementwise("ktanh64_f32", x, out, lut, stream, _F32_VIEWS)


def ksigmoid64(x, out=None, lut=None, stream=None):
    return _elementwise("ksigmoid64", x, out, lut, stream, _BF16_VIEWS)


def kswish64(x, out=None, lut=None, stream=None):
    return _elementwise("kswish64", x, out, lut, stream, _BF16_VIEWS)


def kgelu64(x, out=None, lut=None, stream=None):
    return _elementwise("kgelu64", x, out, lut, stream, _BF16_VIEWS)


def ksigmoid(x, out=None, lut=None, stream=None):
    return _elementwise("ksigmoid", x, out, lut, stream, _BF16_VIEWS)


def kswish(x, out=None, lut=None, stream=None):
    return _elementwise("kswish", x, out, lut, stream, _BF16_VIEWS)


def kgelu(x, out=None, lut=None, stream=None):
    return _elementwise("kgelu", x, out, lut, stream, _BF16_VIEWS)


def ksigmoid_f32(x, out=None, lut=None, stream=None):
    """Sigmoid on a Float32 tensor through the Float32 K-TanH."""
    return _elementwise("ksigmoid_f32", x, out, lut, stream, (torch.float32,))


def kswish_f32(x, out=None, lut=None, stream=None):
    return _elementwise("kswish_f32", x, out, lut, stream, (torch.float32,))


def kgelu_f32(x, out=None, lut=None, stream=None):
    return _elementwise("kgelu_f32", x, out, lut, stream, (torch.float32,))


def ksigmoid64_f32(x, out=None, lut=None, stream=None):
    """Sigmoid on a Float32 tensor through the Float32 K-TanH with a 64-interval table."""
    return _elementwise("ksigmoid64_f32", x, out, lut, stream, (torch.float32,))


def kswish64_f32(x, out=None, lut=None, stream=None):
    return _elementwise("kswish64_f32", x, out, lut, stream, (torch.float32,))


def kgelu64_f32(x, out=None, lut=None, stream=None):
    return _elementwise("kgelu64_f32", x, out, lut, stream, (torch.float32,))


def ktanh_f32_to_bf16(x, out=None, lut=None, stream=None):
    """Float32 tensor in, K-TanH of its BFloat16 rounding out (a bfloat16 tensor unless given)."""
    _check(x, _F32_VIEWS, "in")
    if out is None:
        out = torch.empty(x.shape, dtype=torch.bfloat16, device=x.device)
    _check(out, _BF16_VIEWS, "out")
    if out.numel() != x.numel():
        raise ValueError("in and out differ in size")
    st = load_library().ktanh_f32_to_bf16(x.data_ptr(), out.data_ptr(), x.numel(), _lut_arg(lut),
                                          _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, "ktanh_f32_to_bf16")
    return out


def klstm_cell64(gates, c_in, c_out=None, h_out=None, lut=None, stream=None):
    """``klstm_cell`` with a 64-interval table (``KtanhLut64``; None = the fitted one)."""
    return klstm_cell(gates, c_in, c_out, h_out, lut, stream, _entry="klstm_cell64")


def klstm_cell(gates, c_in, c_out=None, h_out=None, lut=None, stream=None, _entry="klstm_cell"):
    """LSTM-cell element-wise step(s).  gates [T, B, 4H] BFloat16 (i|f|g|o), c_in [B, H] Float32.

    Returns (c_out [B, H] Float32, h_out [T, B, H] in the dtype of ``gates``).
    """
    _check(gates, _BF16_VIEWS, "gates")
    _check(c_in, (torch.float32,), "c_in")
    if gates.dim() != 3 or c_in.dim() != 2:
        raise ValueError("gates must be [T, B, 4H] and c_in [B, H]")
    T, B, H4 = gates.shape
    H = H4 // 4
    if H4 != 4 * H or tuple(c_in.shape) != (B, H):
        raise ValueError("gates [T, B, 4H] and c_in [B, H] do not agree")
    if c_out is None:
        c_out = torch.empty_like(c_in)
    if h_out is None:
        h_out = torch.empty((T, B, H), dtype=gates.dtype, device=gates.device)
    _check(c_out, (torch.float32,), "c_out")
    _check(h_out, _BF16_VIEWS, "h_out")
    if tuple(c_out.shape) != (B, H) or tuple(h_out.shape) != (T, B, H):
        raise ValueError("c_out must be [B, H] and h_out [T, B, H]")
    st = getattr(load_library(), _entry)(gates.data_ptr(), c_in.data_ptr(), c_out.data_ptr(),
                                         h_out.data_ptr(), T, B, H, _lut_arg(lut),
                                         _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, _entry)
    return c_out, h_out


def _backward(name, dy, fwd, dx, stream):
    _check(dy, _BF16_VIEWS, "dy")
    _check(fwd, _BF16_VIEWS, "forward output")
    if dx is None:
        dx = torch.empty_like(dy)
    _check(dx, _BF16_VIEWS, "dx")
    if not (dy.numel() == fwd.numel() == dx.numel()):
        raise ValueError("dy, the forward output and dx differ in size")
    st = getattr(load_library(), name)(dy.data_ptr(), fwd.data_ptr(), dx.data_ptr(), dy.numel(),
                                       _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)
    return dx


def ktanh_bf16_backward(dy, y, dx=None, stream=None):
    """dx = dy * (1 - y^2) from the forward K-TanH output y (BFloat16 tensors)."""
    return _backward("ktanh_bf16_backward", dy, y, dx, stream)


def ksigmoid_backward(dy, s, dx=None, stream=None):
    """dx = dy * s * (1 - s) from the forward Sigmoid output s (BFloat16 tensors)."""
    return _backward("ksigmoid_backward", dy, s, dx, stream)


def _backward_from_input(name, dy, x, dx, lut, stream):
    _check(dy, _BF16_VIEWS, "dy")
    _check(x, _BF16_VIEWS, "x")
    if dx is None:
        dx = torch.empty_like(dy)
    _check(dx, _BF16_VIEWS, "dx")
    if not (dy.numel() == x.numel() == dx.numel()):
        raise ValueError("dy, x and dx differ in size")
    st = getattr(load_library(), name)(dy.data_ptr(), x.data_ptr(), dx.data_ptr(), dy.numel(),
                                       _lut_arg(lut), _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)
    return dx


def kswish_backward(dy, x, dx=None, lut=None, stream=None):
    """dx = dy * (s + x*s*(1 - s)), s = Sigmoid(x) through K-TanH, from the forward input x."""
    return _backward_from_input("kswish_backward", dy, x, dx, lut, stream)


def kgelu_backward(dy, x, dx=None, lut=None, stream=None):
    """dx = dy * GELU'(x) of the tanh form with K-TanH inside, from the forward input x."""
    return _backward_from_input("kgelu_backward", dy, x, dx, lut, stream)


def kswish64_backward(dy, x, dx=None, lut=None, stream=None):
    """``kswish_backward`` with a 64-interval table (``KtanhLut64``; None = the fitted one)."""
    return _backward_from_input("kswish64_backward", dy, x, dx, lut, stream)


def kgelu64_backward(dy, x, dx=None, lut=None, stream=None):
    """``kgelu_backward`` with a 64-interval table (``KtanhLut64``; None = the fitted one)."""
    return _backward_from_input("kgelu64_backward", dy, x, dx, lut, stream)


def _backward_f32(name, dy, v, dx, lut, stream, with_lut):
    for t, what in ((dy, "dy"), (v, "the second input")):
        _check(t, (torch.float32,), what)
    if dx is None:
        dx = torch.empty_like(dy)
    _check(dx, (torch.float32,), "dx")
    if not (dy.numel() == v.numel() == dx.numel()):
        raise ValueError("dy, the second input and dx differ in size")
    args = [dy.data_ptr(), v.data_ptr(), dx.data_ptr(), dy.numel()]
    if with_lut:
        args.append(_lut_arg(lut))
    st = getattr(load_library(), name)(*args, _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, name)
    return dx


def ktanh_f32_backward(dy, y, dx=None, stream=None):
    """dx = dy * (1 - y^2) on Float32 tensors; y = the forward ktanh_f32 output viewed as Float32."""
    return _backward_f32("ktanh_f32_backward", dy, y, dx, None, stream, False)


def ksigmoid_f32_backward(dy, s, dx=None, stream=None):
    """dx = dy * s * (1 - s) on Float32 tensors."""
    return _backward_f32("ksigmoid_f32_backward", dy, s, dx, None, stream, False)


def kswish_f32_backward(dy, x, dx=None, lut=None, stream=None):
    """dx = dy * Swish'(x) on Float32 tensors, from the forward input x."""
    return _backward_f32("kswish_f32_backward", dy, x, dx, lut, stream, True)


def kgelu_f32_backward(dy, x, dx=None, lut=None, stream=None):
    """dx = dy * GELU'(x) on Float32 tensors, from the forward input x."""
    return _backward_f32("kgelu_f32_backward", dy, x, dx, lut, stream, True)


def kswish64_f32_backward(dy, x, dx=None, lut=None, stream=None):
    """``kswish_f32_backward`` with a 64-interval table (``KtanhLut64``; None = the fitted one)."""
    return _backward_f32("kswish64_f32_backward", dy, x, dx, lut, stream, True)


def kgelu64_f32_backward(dy, x, dx=None, lut=None, stream=None):
    """``kgelu_f32_backward`` with a 64-interval table (``KtanhLut64``; None = the fitted one)."""
    return _backward_f32("kgelu64_f32_backward", dy, x, dx, lut, stream, True)


def klstm_cell64_backward(gates, c_prev, dh, dc_next, dgates=None, dc_prev=None, lut=None, stream=None):
    """``klstm_cell_backward`` with a 64-interval table (``KtanhLut64``; None = the fitted one)."""
    return klstm_cell_backward(gates, c_prev, dh, dc_next, dgates, dc_prev, lut, stream,
                               _entry="klstm_cell64_backward")


def klstm_cell_backward(gates, c_prev, dh, dc_next, dgates=None, dc_prev=None, lut=None, stream=None,
                        _entry="klstm_cell_backward"):
    """One LSTM-cell step backwards.  gates [B, 4H] BFloat16, c_prev and dc_next [B, H] Float32,
    dh [B, H] BFloat16.  Returns (dgates [B, 4H], dc_prev [B, H])."""
    _check(gates, _BF16_VIEWS, "gates")
    _check(dh, _BF16_VIEWS, "dh")
    _check(c_prev, (torch.float32,), "c_prev")
    _check(dc_next, (torch.float32,), "dc_next")
    if gates.dim() != 2:
        raise ValueError("gates must be [B, 4H]")
    B, H4 = gates.shape
    H = H4 // 4
    if H4 != 4 * H or not (tuple(c_prev.shape) == tuple(dh.shape) == tuple(dc_next.shape) == (B, H)):
        raise ValueError("gates [B, 4H], c_prev, dh, dc_next [B, H] do not agree")
    if dgates is None:
        dgates = torch.empty_like(gates)
    if dc_prev is None:
        dc_prev = torch.empty_like(c_prev)
    _check(dgates, _BF16_VIEWS, "dgates")
    _check(dc_prev, (torch.float32,), "dc_prev")
    if tuple(dgates.shape) != (B, H4) or tuple(dc_prev.shape) != (B, H):
        raise ValueError("dgates must be [B, 4H] and dc_prev [B, H]")
    st = getattr(load_library(), _entry)(gates.data_ptr(), c_prev.data_ptr(), dh.data_ptr(),
                                         dc_next.data_ptr(), dgates.data_ptr(), dc_prev.data_ptr(),
                                         B, H, _lut_arg(lut), _stream_handle(stream))
    if st != 0:
        raise KtanhError(st, _entry)
    return dgates, dc_prev
