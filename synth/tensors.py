"""Seeded Q/K/V generators, rounded to bf16 (round-to-nearest-even).

Values are N(0,1) float32 draws from numpy's PCG64, then rounded to the nearest bf16.
Arrays are returned as uint16 bit patterns (what the device buffers hold) and can be
widened back to float32 exactly with `bf16_bits_to_f32` (what a CPU checker reads).
"""

from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even; NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32, exact."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def normal_bf16(shape, seed: int, chunk_elems: int = 1 << 24) -> np.ndarray:
    """N(0,1) draws rounded to bf16, returned as uint16 bits with the given shape.

    Drawn in chunks along the flattened array so the float32 staging buffer stays small;
    the stream is one PCG64 generator, so the result does not depend on `chunk_elems`
    only if chunks are consumed in order -- which they are.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    pos = 0
    while pos < n:
        m = min(chunk_elems, n - pos)
        out[pos:pos + m] = f32_to_bf16_bits(rng.standard_normal(m, dtype=np.float32))
        pos += m
    return out.reshape(shape)


def qkv_for_config(cfg: int, B: int, H: int, Nq: int, Nk: int, d: int):
    """Q [B,H,Nq,d], K and V [B,H,Nk,d] as bf16 bits; seeds 1000*cfg + {0,1,2}."""
    q = normal_bf16((B, H, Nq, d), 1000 * cfg + 0)
    k = normal_bf16((B, H, Nk, d), 1000 * cfg + 1)
    v = normal_bf16((B, H, Nk, d), 1000 * cfg + 2)
    return q, k, v
