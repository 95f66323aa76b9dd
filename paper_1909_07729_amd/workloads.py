"""Seeded synthetic inputs for the K-TanH kernels.

Holds no part of the method: it only draws numbers and stores them as BFloat16
or Float32 bit patterns.  Both the GPU tests and the CPU reference read their
inputs from here, so the two always see the same bytes.

The tensors stand in for the activations of the paper's GNMT (LSTM) training
run and for a transformer MLP: same shapes and value spread, no dataset.
"""
from __future__ import annotations

import numpy as np

# shapes of the named workloads
LSTM_GATES_SHAPE = (50, 128, 4096)        # [seq, batch, 4 x hidden 1024]
F32_COUNT = 1 << 28
MLP_SHAPE = (8192, 16384)                 # transformer-MLP pre-activations
LSTM_CELL_T, LSTM_CELL_B, LSTM_CELL_H = 64, 256, 2048

SEED_LSTM_GATES = 190902
SEED_F32 = 190903
SEED_MLP = 190904
SEED_CELL_GATES = 190905
SEED_CELL_STATE = 190906


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Float32 array -> BFloat16 bit patterns (uint16), round to nearest even.

    Input preparation only (the draws below are never NaN).
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """BFloat16 bit patterns (uint16) -> Float32 values (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def all_bf16_patterns() -> np.ndarray:
    """Every BFloat16 bit pattern, 0x0000..0xFFFF in index order."""
    return np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)


def _normal_bf16(seed: int, count: int, sigma: float, chunk: int = 1 << 24) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty(count, dtype=np.uint16)
    for lo in range(0, count, chunk):
        m = min(chunk, count - lo)
        draw = rng.standard_normal(m, dtype=np.float32) * np.float32(sigma)
        out[lo:lo + m] = f32_to_bf16_bits(draw)
    return out


def lstm_gate_preactivations(count: int | None = None, seed: int = SEED_LSTM_GATES) -> np.ndarray:
    """BFloat16 bits ~ N(0, 1.5^2); full size = 50 x 128 x 4096 values (flat)."""
    if count is None:
        count = int(np.prod(LSTM_GATES_SHAPE))
    return _normal_bf16(seed, count, 1.5)


def mlp_preactivations(count: int | None = None, seed: int = SEED_MLP) -> np.ndarray:
    """BFloat16 bits ~ N(0, 1); full size = 8192 x 16384 values (flat)."""
    if count is None:
        count = int(np.prod(MLP_SHAPE))
    return _normal_bf16(seed, count, 1.0)


def f32_mixture(count: int = F32_COUNT, seed: int = SEED_F32, chunk: int = 1 << 24) -> np.ndarray:
    """Float32 bit patterns (uint32): uniform in [-8, 8), 5 % replaced by N(0, 0.01^2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty(count, dtype=np.uint32)
    for lo in range(0, count, chunk):
        m = min(chunk, count - lo)
        wide = rng.random(m, dtype=np.float32) * np.float32(16.0) - np.float32(8.0)
        pick = rng.random(m, dtype=np.float32) < np.float32(0.05)
        small = rng.standard_normal(m, dtype=np.float32) * np.float32(0.01)
        out[lo:lo + m] = np.where(pick, small, wide).astype(np.float32).view(np.uint32)
    return out


def lstm_cell_inputs(T: int = LSTM_CELL_T, B: int = LSTM_CELL_B, H: int = LSTM_CELL_H,
                     seed_gates: int = SEED_CELL_GATES, seed_state: int = SEED_CELL_STATE):
    """(gates uint16 [T, B, 4H] ~ N(0, 2^2) as BFloat16 bits, c0 float32 [B, H] ~ N(0, 1))."""
    gates = _normal_bf16(seed_gates, T * B * 4 * H, 2.0).reshape(T, B, 4 * H)
    rng = np.random.Generator(np.random.PCG64(seed_state))
    c0 = rng.standard_normal((B, H), dtype=np.float32)
    return gates, c0


def edge_bf16_patterns() -> np.ndarray:
    """A short list of BFloat16 corner patterns (zeros, subnormals, thresholds, Inf, NaN)."""
    pos = [0x0000, 0x0001, 0x007F, 0x0080, 0x00FF, 0x0100, 0x3E7F, 0x3E80, 0x3E81, 0x3EFF, 0x3F00,
           0x3F7F, 0x3F80, 0x3FFF, 0x4000, 0x406F, 0x4070, 0x407F, 0x4080, 0x4081, 0x7F7F, 0x7F80,
           0x7F81, 0x7FBF, 0x7FC0, 0x7FFF]
    return np.array(pos + [v | 0x8000 for v in pos], dtype=np.uint16)
