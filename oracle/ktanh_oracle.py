"""ctypes front-end of the K-TanH reference oracle (``ktanh_oracle.c``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import this; the GPU library never does.  Everything here
works on host numpy arrays; nothing here touches a GPU, and nothing here is
shared with the HIP code.

``build()`` compiles the C file with gcc (no fused multiply-add, no fast-math);
every other function loads the built library on first use.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ktanh_oracle.c")
_LIB = os.path.join(_HERE, "libktanh_oracle.so")

N_INTERVALS = 32


class OracleLut(ctypes.Structure):
    """The three 32-entry parameter tables of Table 1, indexed by t."""

    _fields_ = [
        ("E", ctypes.c_uint8 * N_INTERVALS),
        ("r", ctypes.c_uint8 * N_INTERVALS),
        ("b", ctypes.c_int8 * N_INTERVALS),
    ]

    def as_tuples(self):
        return [(int(self.E[t]), int(self.r[t]), int(self.b[t])) for t in range(N_INTERVALS)]

    @classmethod
    def from_tuples(cls, rows):
        lut = cls()
        for t, (E, r, b) in enumerate(rows):
            lut.E[t], lut.r[t], lut.b[t] = E, r, b
        return lut


class OracleLut64(ctypes.Structure):
    """64-interval tables: index t = (2 LSBs of E_i) << 4 | (4 MSBs of M_i)."""

    _fields_ = [
        ("E", ctypes.c_uint8 * 64),
        ("r", ctypes.c_uint8 * 64),
        ("b", ctypes.c_int8 * 64),
    ]

    def as_tuples(self):
        return [(int(self.E[t]), int(self.r[t]), int(self.b[t])) for t in range(64)]

    @classmethod
    def from_tuples(cls, rows):
        lut = cls()
        for t, (E, r, b) in enumerate(rows):
            lut.E[t], lut.r[t], lut.b[t] = E, r, b
        return lut


def build(force: bool = False) -> str:
    """Compile the oracle; returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = [
            "gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
            "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm",
        ]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lp = ctypes.POINTER(OracleLut)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        lib.oracle_table1.argtypes = [lp]
        lib.oracle_fit_lut.argtypes = [lp]
        lib.oracle_fit_lut_bmin0.argtypes = [lp]
        lib.oracle_fit_lut_bmin0.restype = None
        for name in ("oracle_ktanh_bf16", "oracle_ktanh_f32", "oracle_ksigmoid", "oracle_kswish",
                     "oracle_kgelu"):
            getattr(lib, name).argtypes = [vp, vp, sz, lp]
            getattr(lib, name).restype = None
        lib.oracle_klstm_cell.argtypes = [vp, vp, vp, vp, sz, sz, sz, lp]
        lib.oracle_klstm_cell.restype = None
        for name in ("oracle_ksigmoid_f32", "oracle_kswish_f32", "oracle_kgelu_f32",
                     "oracle_ktanh_f32_to_bf16"):
            getattr(lib, name).argtypes = [vp, vp, sz, lp]
            getattr(lib, name).restype = None
        for name in ("oracle_ksigmoid64_f32", "oracle_kswish64_f32", "oracle_kgelu64_f32"):
            getattr(lib, name).argtypes = [vp, vp, sz, ctypes.POINTER(OracleLut64)]
            getattr(lib, name).restype = None
        for name in ("oracle_ktanh_backward", "oracle_ksigmoid_backward"):
            getattr(lib, name).argtypes = [vp, vp, vp, sz]
            getattr(lib, name).restype = None
        for name in ("oracle_ktanh_f32_backward", "oracle_ksigmoid_f32_backward"):
            getattr(lib, name).argtypes = [vp, vp, vp, sz]
            getattr(lib, name).restype = None
        for name in ("oracle_kswish_f32_backward", "oracle_kgelu_f32_backward"):
            getattr(lib, name).argtypes = [vp, vp, vp, sz, lp]
            getattr(lib, name).restype = None
        for name in ("oracle_kswish_backward", "oracle_kgelu_backward"):
            getattr(lib, name).argtypes = [vp, vp, vp, sz, lp]
            getattr(lib, name).restype = None
        lib.oracle_klstm_cell_backward.argtypes = [vp, vp, vp, vp, vp, vp, sz, sz, lp]
        lib.oracle_klstm_cell_backward.restype = None
        for name in ("oracle_kswish64_backward", "oracle_kgelu64_backward",
                     "oracle_kswish64_f32_backward", "oracle_kgelu64_f32_backward"):
            getattr(lib, name).argtypes = [vp, vp, vp, sz, ctypes.POINTER(OracleLut64)]
            getattr(lib, name).restype = None
        lib.oracle_klstm_cell64_backward.argtypes = [vp, vp, vp, vp, vp, vp, sz, sz,
                                                     ctypes.POINTER(OracleLut64)]
        lib.oracle_klstm_cell64_backward.restype = None
        for name in ("oracle_kpade32", "oracle_kpade78"):
            getattr(lib, name).argtypes = [vp, vp, sz]
            getattr(lib, name).restype = None
        lib.oracle_pade_coefficients.argtypes = [ctypes.c_int, vp, vp]
        lib.oracle_pade_coefficients.restype = None
        for name in ("oracle_ktaylor2", "oracle_ktaylor3"):
            getattr(lib, name).argtypes = [vp, vp, sz]
            getattr(lib, name).restype = None
        lib.oracle_taylor_coefficients.argtypes = [vp]
        lib.oracle_taylor_coefficients.restype = None
        lp64 = ctypes.POINTER(OracleLut64)
        lib.oracle_fit_lut64.argtypes = [lp64]
        for name in ("oracle_ktanh64_bf16", "oracle_ktanh64_f32", "oracle_ksigmoid64", "oracle_kswish64",
                     "oracle_kgelu64"):
            getattr(lib, name).argtypes = [vp, vp, sz, lp64]
            getattr(lib, name).restype = None
        lib.oracle_klstm_cell64.argtypes = [vp, vp, vp, vp, sz, sz, sz, lp64]
        lib.oracle_klstm_cell64.restype = None
        _lib = lib
    return _lib


def table1() -> OracleLut:
    """Table 1 as printed in the paper."""
    lut = OracleLut()
    _load().oracle_table1(ctypes.byref(lut))
    return lut


def fit_lut() -> OracleLut:
    """Parameters regenerated by the optimisation of Section 2.4 (Steps 1-3)."""
    lut = OracleLut()
    _load().oracle_fit_lut(ctypes.byref(lut))
    return lut


def fit_lut_bmin0() -> OracleLut:
    """The ablation's sub-optimal parameters: the same optimisation with b_min = 0."""
    lut = OracleLut()
    _load().oracle_fit_lut_bmin0(ctypes.byref(lut))
    return lut


def fit_lut64() -> OracleLut64:
    """64-interval parameters from the same optimisation (4 mantissa bits in the index)."""
    lut = OracleLut64()
    _load().oracle_fit_lut64(ctypes.byref(lut))
    return lut


def ktanh64_bf16(x_bits, lut64=None):
    """Algorithm 1 with 64-interval tables on BFloat16 bit patterns."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    out = np.empty_like(x)
    lut64 = fit_lut64() if lut64 is None else lut64
    _load().oracle_ktanh64_bf16(x.ctypes.data, out.ctypes.data, x.size, ctypes.byref(lut64))
    return out


def ktanh64_f32(x_bits, lut64=None):
    """Algorithm 1 with 64-interval tables on Float32 bit patterns."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint32)
    out = np.empty_like(x)
    lut64 = fit_lut64() if lut64 is None else lut64
    _load().oracle_ktanh64_f32(x.ctypes.data, out.ctypes.data, x.size, ctypes.byref(lut64))
    return out


def _elementwise64(name, x, lut64):
    x = np.ascontiguousarray(x, dtype=np.uint16)
    out = np.empty_like(x)
    lut64 = fit_lut64() if lut64 is None else lut64
    getattr(_load(), name)(x.ctypes.data, out.ctypes.data, x.size, ctypes.byref(lut64))
    return out


def ksigmoid64(x_bits, lut64=None):
    """Sigmoid through the 64-interval K-TanH, BFloat16 bits in and out."""
    return _elementwise64("oracle_ksigmoid64", x_bits, lut64)


def kswish64(x_bits, lut64=None):
    return _elementwise64("oracle_kswish64", x_bits, lut64)


def kgelu64(x_bits, lut64=None):
    return _elementwise64("oracle_kgelu64", x_bits, lut64)


def klstm_cell64(gates_bits, c_in, lut64=None):
    """LSTM-cell non-linearities over T steps with 64-interval tables; as klstm_cell."""
    gates = np.ascontiguousarray(gates_bits, dtype=np.uint16)
    c_in = np.ascontiguousarray(c_in, dtype=np.float32)
    T, B, H4 = gates.shape
    H = H4 // 4
    assert H4 == 4 * H and c_in.shape == (B, H)
    c_out = np.empty_like(c_in)
    h_out = np.empty((T, B, H), dtype=np.uint16)
    lut64 = fit_lut64() if lut64 is None else lut64
    _load().oracle_klstm_cell64(gates.ctypes.data, c_in.ctypes.data, c_out.ctypes.data,
                                h_out.ctypes.data, T, B, H, ctypes.byref(lut64))
    return c_out, h_out


def _elementwise(name, x, dtype, lut):
    x = np.ascontiguousarray(x, dtype=dtype)
    out = np.empty_like(x)
    lut = table1() if lut is None else lut
    getattr(_load(), name)(x.ctypes.data, out.ctypes.data, x.size, ctypes.byref(lut))
    return out


def ktanh_bf16(x_bits, lut=None):
    """Algorithm 1 on BFloat16 bit patterns (uint16 in, uint16 out)."""
    return _elementwise("oracle_ktanh_bf16", x_bits, np.uint16, lut)


def ktanh_f32(x_bits, lut=None):
    """Algorithm 1 on Float32 bit patterns (uint32 in, uint32 out)."""
    return _elementwise("oracle_ktanh_f32", x_bits, np.uint32, lut)


def ksigmoid(x_bits, lut=None):
    """Sigmoid through K-TanH, BFloat16 bits in and out."""
    return _elementwise("oracle_ksigmoid", x_bits, np.uint16, lut)


def kswish(x_bits, lut=None):
    """Swish through K-TanH, BFloat16 bits in and out."""
    return _elementwise("oracle_kswish", x_bits, np.uint16, lut)


def kgelu(x_bits, lut=None):
    """GELU (tanh form, a = 0.044715) through K-TanH, BFloat16 bits in and out."""
    return _elementwise("oracle_kgelu", x_bits, np.uint16, lut)


def _f32_op(name, x, out_dtype, lut):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=out_dtype)
    lut = table1() if lut is None else lut
    getattr(_load(), name)(x.ctypes.data, out.ctypes.data, x.size, ctypes.byref(lut))
    return out


def ksigmoid_f32(x, lut=None):
    """Sigmoid through the Float32 K-TanH; float32 values in and out."""
    return _f32_op("oracle_ksigmoid_f32", x, np.float32, lut)


def kswish_f32(x, lut=None):
    return _f32_op("oracle_kswish_f32", x, np.float32, lut)


def kgelu_f32(x, lut=None):
    return _f32_op("oracle_kgelu_f32", x, np.float32, lut)


def _f32_op64(name, x, lut64):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.float32)
    lut64 = fit_lut64() if lut64 is None else lut64
    getattr(_load(), name)(x.ctypes.data, out.ctypes.data, x.size, ctypes.byref(lut64))
    return out


def ksigmoid64_f32(x, lut64=None):
    """Sigmoid through the Float32 K-TanH on 64-interval tables; float32 values in and out."""
    return _f32_op64("oracle_ksigmoid64_f32", x, lut64)


def kswish64_f32(x, lut64=None):
    return _f32_op64("oracle_kswish64_f32", x, lut64)


def kgelu64_f32(x, lut64=None):
    return _f32_op64("oracle_kgelu64_f32", x, lut64)


def ktanh_f32_to_bf16(x, lut=None):
    """float32 values in, K-TanH of their BFloat16 rounding out (uint16 bit patterns)."""
    return _f32_op("oracle_ktanh_f32_to_bf16", x, np.uint16, lut)


def klstm_cell(gates_bits, c_in, lut=None):
    """LSTM-cell non-linearities over T steps.

    gates_bits: uint16 [T, B, 4H] (i|f|g|o blocks); c_in: float32 [B, H].
    Returns (c_out float32 [B, H], h_out uint16 [T, B, H]).
    """
    gates = np.ascontiguousarray(gates_bits, dtype=np.uint16)
    c_in = np.ascontiguousarray(c_in, dtype=np.float32)
    T, B, H4 = gates.shape
    H = H4 // 4
    assert H4 == 4 * H and c_in.shape == (B, H)
    c_out = np.empty_like(c_in)
    h_out = np.empty((T, B, H), dtype=np.uint16)
    lut = table1() if lut is None else lut
    _load().oracle_klstm_cell(gates.ctypes.data, c_in.ctypes.data, c_out.ctypes.data,
                              h_out.ctypes.data, T, B, H, ctypes.byref(lut))
    return c_out, h_out


def _pade(name, x_bits):
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    out = np.empty_like(x)
    getattr(_load(), name)(x.ctypes.data, out.ctypes.data, x.size)
    return out


def kpade32(x_bits):
    """The Pade[3/2] approximant of TanH, BFloat16 bits in and out."""
    return _pade("oracle_kpade32", x_bits)


def kpade78(x_bits):
    """The Pade[7/8] approximant of TanH, BFloat16 bits in and out."""
    return _pade("oracle_kpade78", x_bits)


def pade_coefficients(which):
    """(numerator, denominator) coefficient lists of x^0, x^1, ... for which = 32 or 78."""
    p, q = (3, 2) if which == 32 else (7, 8)
    num, den = np.zeros(p + 1), np.zeros(q + 1)
    _load().oracle_pade_coefficients(which, num.ctypes.data, den.ctypes.data)
    return num.tolist(), den.tolist()


def ktaylor2(x_bits):
    """Piecewise Taylor polynomial of degree 2 about the midpoints of K-TanH's intervals, BFloat16 bits."""
    return _pade("oracle_ktaylor2", x_bits)


def ktaylor3(x_bits):
    """The same of degree 3."""
    return _pade("oracle_ktaylor3", x_bits)


def taylor_coefficients():
    """[32, 4] Float32: for Table 1's index t, the coefficients of (|x| - a_t)^0 .. ^3."""
    c = np.zeros((32, 4), dtype=np.float32)
    _load().oracle_taylor_coefficients(c.ctypes.data)
    return c


def _backward(name, dy_bits, fwd_bits):
    dy = np.ascontiguousarray(dy_bits, dtype=np.uint16)
    fwd = np.ascontiguousarray(fwd_bits, dtype=np.uint16)
    assert dy.shape == fwd.shape
    dx = np.empty_like(dy)
    getattr(_load(), name)(dy.ctypes.data, fwd.ctypes.data, dx.ctypes.data, dy.size)
    return dx


def ktanh_backward(dy_bits, y_bits):
    """dx = dy * (1 - y^2) from the forward K-TanH output y; BFloat16 bits throughout."""
    return _backward("oracle_ktanh_backward", dy_bits, y_bits)


def ksigmoid_backward(dy_bits, s_bits):
    """dx = dy * s * (1 - s) from the forward Sigmoid output s; BFloat16 bits throughout."""
    return _backward("oracle_ksigmoid_backward", dy_bits, s_bits)


def _backward_from_input(name, dy_bits, x_bits, lut, wide=False):
    dy = np.ascontiguousarray(dy_bits, dtype=np.uint16)
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    assert dy.shape == x.shape
    dx = np.empty_like(dy)
    if lut is None:
        lut = fit_lut64() if wide else table1()
    getattr(_load(), name)(dy.ctypes.data, x.ctypes.data, dx.ctypes.data, dy.size, ctypes.byref(lut))
    return dx


def kswish_backward(dy_bits, x_bits, lut=None):
    """dx = dy * (s + x*s*(1 - s)), s = Sigmoid(x) through K-TanH, from the forward INPUT x."""
    return _backward_from_input("oracle_kswish_backward", dy_bits, x_bits, lut)


def kgelu_backward(dy_bits, x_bits, lut=None):
    """dx = dy * GELU'(x) of the tanh form with K-TanH inside, from the forward INPUT x."""
    return _backward_from_input("oracle_kgelu_backward", dy_bits, x_bits, lut)


def kswish64_backward(dy_bits, x_bits, lut64=None):
    """kswish_backward with a 64-interval table (None = the fitted one)."""
    return _backward_from_input("oracle_kswish64_backward", dy_bits, x_bits, lut64, wide=True)


def kgelu64_backward(dy_bits, x_bits, lut64=None):
    """kgelu_backward with a 64-interval table (None = the fitted one)."""
    return _backward_from_input("oracle_kgelu64_backward", dy_bits, x_bits, lut64, wide=True)


def _f32_backward(name, dy, v, lut=None, with_lut=False, wide=False):
    dy = np.ascontiguousarray(dy, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    assert dy.shape == v.shape
    dx = np.empty_like(dy)
    if with_lut:
        if lut is None:
            lut = fit_lut64() if wide else table1()
        getattr(_load(), name)(dy.ctypes.data, v.ctypes.data, dx.ctypes.data, dy.size, ctypes.byref(lut))
    else:
        getattr(_load(), name)(dy.ctypes.data, v.ctypes.data, dx.ctypes.data, dy.size)
    return dx


def ktanh_f32_backward(dy, y):
    """dx = dy * (1 - y^2), float32 throughout; y = the forward Float32 K-TanH output."""
    return _f32_backward("oracle_ktanh_f32_backward", dy, y)


def ksigmoid_f32_backward(dy, s):
    """dx = dy * s * (1 - s), float32 throughout; s = the forward ksigmoid_f32 output."""
    return _f32_backward("oracle_ksigmoid_f32_backward", dy, s)


def kswish_f32_backward(dy, x, lut=None):
    """dx = dy * Swish'(x) from the forward input x, float32 throughout."""
    return _f32_backward("oracle_kswish_f32_backward", dy, x, lut, True)


def kgelu_f32_backward(dy, x, lut=None):
    """dx = dy * GELU'(x) from the forward input x, float32 throughout."""
    return _f32_backward("oracle_kgelu_f32_backward", dy, x, lut, True)


def kswish64_f32_backward(dy, x, lut64=None):
    """kswish_f32_backward with a 64-interval table (None = the fitted one)."""
    return _f32_backward("oracle_kswish64_f32_backward", dy, x, lut64, True, wide=True)


def kgelu64_f32_backward(dy, x, lut64=None):
    """kgelu_f32_backward with a 64-interval table (None = the fitted one)."""
    return _f32_backward("oracle_kgelu64_f32_backward", dy, x, lut64, True, wide=True)


def klstm_cell64_backward(gates_bits, c_prev, dh_bits, dc_next, lut64=None):
    """klstm_cell_backward with a 64-interval table (None = the fitted one)."""
    return klstm_cell_backward(gates_bits, c_prev, dh_bits, dc_next,
                               fit_lut64() if lut64 is None else lut64,
                               _entry="oracle_klstm_cell64_backward")


def klstm_cell_backward(gates_bits, c_prev, dh_bits, dc_next, lut=None,
                        _entry="oracle_klstm_cell_backward"):
    """One LSTM-cell step backwards.  gates uint16 [B, 4H], c_prev/dc_next float32 [B, H],
    dh uint16 [B, H].  Returns (dgates uint16 [B, 4H], dc_prev float32 [B, H])."""
    gates = np.ascontiguousarray(gates_bits, dtype=np.uint16)
    c_prev = np.ascontiguousarray(c_prev, dtype=np.float32)
    dh = np.ascontiguousarray(dh_bits, dtype=np.uint16)
    dc_next = np.ascontiguousarray(dc_next, dtype=np.float32)
    B, H4 = gates.shape
    H = H4 // 4
    assert H4 == 4 * H and c_prev.shape == (B, H) == dh.shape == dc_next.shape
    dgates = np.empty_like(gates)
    dc_prev = np.empty_like(c_prev)
    lut = table1() if lut is None else lut
    getattr(_load(), _entry)(gates.ctypes.data, c_prev.ctypes.data, dh.ctypes.data,
                             dc_next.ctypes.data, dgates.ctypes.data, dc_prev.ctypes.data,
                             B, H, ctypes.byref(lut))
    return dgates, dc_prev
