"""Seeded bf16-valued GEMM operands (inputs only)."""
import numpy as np


def bf16_round(x32: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result kept as float32."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def bf16_bits(x32: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable float32 values."""
    return (np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def operands(M: int, N: int, K: int, seed: int):
    """A [M, K] and B [N, K], uniform in [-1, 1), rounded to bf16, as float32 arrays."""
    rng = np.random.default_rng(seed)
    a = bf16_round(rng.uniform(-1, 1, size=(M, K)).astype(np.float32))
    b = bf16_round(rng.uniform(-1, 1, size=(N, K)).astype(np.float32))
    return a, b
