"""Q/K/V generators.  bf16 tensors travel as uint16 bit patterns so numpy can hold them."""
import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns.

    Inputs must be finite (the generators only draw finite normals)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def make_qkv(B: int, H: int, N: int, d: int, seed: int, std: float = 1.0):
    """Q, K, V ~ N(0, std^2) drawn in float32 and rounded to bf16; returns three uint16 [B,H,N,d] arrays."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(3):
        x = rng.standard_normal((B, H, N, d), dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out.append(f32_to_bf16_bits(x))
    return tuple(out)
