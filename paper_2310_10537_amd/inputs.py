"""Seeded synthetic inputs shaped like the paper's transformer workloads.

This module serves both the GPU tests/bench and the CPU reference, and holds
none of the MX arithmetic: it only draws random tensors and narrows them to
bfloat16 storage.  Everything is numpy on the host; bf16 tensors are returned
as uint16 arrays of bit patterns so that both sides consume the same bytes.

The paper's models (GPT-like 20M-1.5B, GPT3-175B, LLaMA-7B; Sections 4.4-4.5)
are not available, so Gaussian weights (std 0.02), Gaussian activations and
gradients, and heavy-tailed Student-t activations with sparse large outliers
stand in for them.
"""
import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 storage (nearest, ties to even); uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (((u >> 16) & 1) + 0x7FFF).astype(np.uint32)) >> 16
    r = np.where(nan, (u >> 16) | 0x0040, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def gaussian_f32(shape, seed: int, std: float = 1.0) -> np.ndarray:
    """i.i.d. N(0, std^2) as float32."""
    return (_rng(seed).standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def gaussian_bf16(shape, seed: int, std: float = 1.0) -> np.ndarray:
    return f32_to_bf16_bits(gaussian_f32(shape, seed, std))


def student_t_f32(shape, seed: int, nu: float = 3.0, outlier_frac: float = 1e-3,
                  outlier_mul: float = 100.0, zero_frac: float = 1e-4) -> np.ndarray:
    """Heavy-tailed activations: Student-t(nu); an independent Bernoulli mask
    multiplies outlier_frac of the entries by outlier_mul; another sets
    zero_frac of them to exact zero."""
    g = _rng(seed)
    x = g.standard_t(nu, size=shape).astype(np.float32)
    out = g.random(shape, dtype=np.float32) < outlier_frac
    x = np.where(out, x * np.float32(outlier_mul), x)
    zero = g.random(shape, dtype=np.float32) < zero_frac
    x = np.where(zero, np.float32(0.0), x)
    return np.ascontiguousarray(x, dtype=np.float32)


def student_t_bf16(shape, seed: int, **kw) -> np.ndarray:
    return f32_to_bf16_bits(student_t_f32(shape, seed, **kw))


def adversarial_f32(rows: int, cols: int, seed: int) -> np.ndarray:
    """Float32 tensor [rows, cols] (cols a multiple of 32) whose 32-blocks cycle
    through the degenerate cases of the cast: all zero, one huge outlier, all
    equal, exact rounding ties, Float32 subnormals, +-Inf, NaN, largest finite,
    negative zero, tiny normals, and plain random data over the full exponent
    range."""
    g = _rng(seed)
    assert cols % 32 == 0
    nblk = rows * cols // 32
    x = np.empty((nblk, 32), dtype=np.float32)
    # random sign / exponent / mantissa over the whole normal range
    bits = g.integers(0, 2**32, size=(nblk, 32), dtype=np.uint64).astype(np.uint32)
    expo = g.integers(1, 255, size=(nblk, 1), dtype=np.uint32)  # per-block exponent centre
    spread = g.integers(0, 12, size=(nblk, 32), dtype=np.uint32)
    e = np.clip(expo.astype(np.int64) - spread.astype(np.int64), 1, 254).astype(np.uint32)
    x[:] = ((bits & 0x807FFFFF) | (e << 23)).view(np.float32)
    kinds = 16
    for b in range(nblk):
        k = b % kinds
        blk = x[b]
        if k == 0:
            blk[:] = 0.0
        elif k == 1:
            blk[:] = g.standard_normal(32).astype(np.float32)
            blk[g.integers(0, 32)] = np.float32(3.0e38)
        elif k == 2:
            blk[:] = np.float32(g.standard_normal()) * np.float32(2.0 ** int(g.integers(-100, 100)))
        elif k == 3:
            # multiples of 1/16 with alternating sign: many exact midpoints
            blk[:] = (g.integers(-64, 65, size=32).astype(np.float32) / np.float32(16.0))
            blk[0] = np.float32(4.0)
        elif k == 4:
            blk[:] = (g.integers(0, 1 << 23, size=32, dtype=np.uint64).astype(np.uint32)
                      | (g.integers(0, 2, size=32, dtype=np.uint64).astype(np.uint32) << 31)).view(np.float32)
        elif k == 5:
            blk[g.integers(0, 32)] = np.float32(np.inf)
        elif k == 6:
            blk[g.integers(0, 32)] = np.float32(-np.inf)
        elif k == 7:
            blk[g.integers(0, 32)] = np.float32(np.nan)
        elif k == 8:
            blk[:] = g.standard_normal(32).astype(np.float32)
            blk[3] = np.finfo(np.float32).max
            blk[4] = -np.finfo(np.float32).max
        elif k == 9:
            blk[::2] = np.float32(-0.0)
        elif k == 10:
            blk[:] = (g.standard_normal(32) * 2.0 ** -125).astype(np.float32)
        elif k == 11:
            # mix of subnormals and one small normal
            blk[:] = (g.integers(0, 1 << 23, size=32, dtype=np.uint64).astype(np.uint32)).view(np.float32)
            blk[7] = np.float32(2.0 ** -126)
        # 12..15: leave the full-range random data
    return np.ascontiguousarray(x.reshape(rows, cols))
