"""Pins for the reference MX dot product (CPU only): brute force in exact
rational arithmetic on tiny operands, exactly known integer results, linearity
in the block scales (Section 4.1's sum over blocks of X_A * X_B * sum a_j b_j),
one-hot operands, NaN propagation, and numpy's matmul on dequantized operands.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2310_10537_amd import inputs

E4M3, E5M2, E3M2, E2M3, E2M1, INT8 = range(6)
BITS = {E4M3: 8, E5M2: 8, E3M2: 6, E2M3: 6, E2M1: 4, INT8: 8}


def unpack(elems, w):
    bits = np.unpackbits(np.ascontiguousarray(elems), axis=-1, bitorder="little")
    bits = bits.reshape(*elems.shape[:-1], -1, w)
    return (bits.astype(np.uint32) << np.arange(w, dtype=np.uint32)).sum(axis=-1).astype(np.uint32)


def pack(codes, w):
    bits = ((codes.astype(np.uint32)[..., None] >> np.arange(w, dtype=np.uint32)) & 1).astype(np.uint8)
    return np.packbits(bits.reshape(*codes.shape[:-1], -1), axis=-1, bitorder="little")


@pytest.mark.parametrize("fa,fb", [(E4M3, E4M3), (E2M1, E3M2), (E3M2, E3M2), (E5M2, E2M3), (INT8, INT8), (E2M1, E2M1)])
@pytest.mark.parametrize("K", [32, 64])
def test_brute_force_blockwise_formula(oracle, fa, fb, K):
    """C = sum over blocks of X_A * X_B * sum_j a_j * b_j, in exact fractions,
    straight from the block structure (scales and codes), not from dequantized
    tensors."""
    M, N = 3, 4
    a = inputs.student_t_f32((M, K), seed=K + fa)
    b = inputs.gaussian_f32((N, K), seed=K + fb + 50, std=0.02)
    ea, sa = oracle.quantize(a, 1, fa)
    eb, sb = oracle.quantize(b, 1, fb)
    ca, cb = unpack(ea, BITS[fa]), unpack(eb, BITS[fb])
    C = oracle.gemm(ea, sa, fa, eb, sb, fb, K)
    for m in range(M):
        for n in range(N):
            tot = Fraction(0)
            for blk in range(K // 32):
                XA = Fraction(2) ** (int(sa[m, blk]) - 127)
                XB = Fraction(2) ** (int(sb[n, blk]) - 127)
                inner = sum(Fraction(oracle.decode(fa, int(ca[m, 32 * blk + j]))) *
                            Fraction(oracle.decode(fb, int(cb[n, 32 * blk + j]))) for j in range(32))
                tot += XA * XB * inner
            assert abs(Fraction(C[m, n]) - tot) <= abs(tot) * Fraction(1, 2**45) + Fraction(1, 2**200)


def test_integer_valued_operands_give_exact_integers(oracle):
    # E2M1 holds 0, 1, 2, 3, 4, 6 exactly at X = 1 (scale byte 127 needs a block max in [4, 8))
    rng = np.random.default_rng(0)
    vals = np.array([0, 1, 2, 3, 4, 6, -1, -2, -3, -4, -6], dtype=np.float32)
    a = rng.choice(vals, (8, 96)).astype(np.float32)
    b = rng.choice(vals, (5, 96)).astype(np.float32)
    a[:, ::32] = 4
    b[:, ::32] = -6
    ea, sa = oracle.quantize(a, 1, E2M1)
    eb, sb = oracle.quantize(b, 1, E2M1)
    assert (sa == 127).all() and (sb == 127).all()
    C, Cabs = oracle.gemm(ea, sa, E2M1, eb, sb, E2M1, 96, want_abs=True)
    ref = a.astype(np.int64) @ b.astype(np.int64).T
    assert np.array_equal(C, ref.astype(np.float64))
    assert np.array_equal(Cabs, (np.abs(a).astype(np.int64) @ np.abs(b).astype(np.int64).T).astype(np.float64))


def test_scale_linearity_per_block(oracle):
    """Adding t to the scale byte of block b of one row of A multiplies exactly
    that block's contribution by 2^t."""
    K = 96
    a = inputs.gaussian_f32((2, K), seed=1)
    b = inputs.gaussian_f32((3, K), seed=2)
    ea, sa = oracle.quantize(a, 1, E4M3)
    eb, sb = oracle.quantize(b, 1, E5M2)
    C0 = oracle.gemm(ea, sa, E4M3, eb, sb, E5M2, K)
    # contribution of block 1 alone: zero the other blocks' elements
    z = ea.copy()
    z[:, :32] = 0
    z[:, 64:] = 0
    part = oracle.gemm(z, sa, E4M3, eb, sb, E5M2, K)
    for t in (1, 5, -3):
        s2 = sa.copy()
        s2[0, 1] = np.uint8(int(sa[0, 1]) + t)
        C1 = oracle.gemm(ea, s2, E4M3, eb, sb, E5M2, K)
        assert np.allclose(C1[0], C0[0] + part[0] * (2.0**t - 1), rtol=1e-13, atol=0)
        assert np.array_equal(C1[1], C0[1])


def test_one_hot_rows_pick_single_elements(oracle):
    K = 64
    b = inputs.student_t_f32((6, K), seed=3)
    eb, sb = oracle.quantize(b, 1, E3M2)
    bd = oracle.dequantize(eb, sb, E3M2, 6, K, 1).astype(np.float64)
    a = np.zeros((K, K), dtype=np.float32)
    np.fill_diagonal(a, 1.0)            # row m of A is the m-th unit vector
    ea, sa = oracle.quantize(a, 1, E2M1)
    C = oracle.gemm(ea, sa, E2M1, eb, sb, E3M2, K)
    assert np.array_equal(C, bd.T)      # C[m, n] = B[n, m]; a transposed operand would fail


@pytest.mark.parametrize("fa,fb", [(E4M3, E4M3), (E2M1, E3M2), (INT8, E2M3)])
def test_against_numpy_matmul_and_entries(oracle, fa, fb):
    M, N, K = 24, 40, 256
    a = inputs.student_t_f32((M, K), seed=5)
    b = inputs.gaussian_f32((N, K), seed=6, std=0.02)
    ea, sa = oracle.quantize(a, 1, fa)
    eb, sb = oracle.quantize(b, 1, fb)
    C, Cabs = oracle.gemm(ea, sa, fa, eb, sb, fb, K, want_abs=True)
    ad = oracle.dequantize(ea, sa, fa, M, K, 1).astype(np.float64)
    bd = oracle.dequantize(eb, sb, fb, N, K, 1).astype(np.float64)
    ref = ad @ bd.T
    assert np.allclose(C, ref, rtol=0, atol=1e-12 * np.abs(ad).sum(1).max() * np.abs(bd).max())
    assert np.allclose(Cabs, np.abs(ad) @ np.abs(bd).T, rtol=1e-12)
    rng = np.random.default_rng(0)
    mi, ni = rng.integers(0, M, 50), rng.integers(0, N, 50)
    Ce, Cae = oracle.gemm_entries(ea, sa, fa, eb, sb, fb, K, mi, ni)
    assert np.array_equal(Ce, C[mi, ni]) and np.array_equal(Cae, Cabs[mi, ni])


def test_nan_propagation(oracle):
    K = 64
    a = inputs.gaussian_f32((4, K), seed=7)
    b = inputs.gaussian_f32((4, K), seed=8)
    ea, sa = oracle.quantize(a, 1, E2M1)
    eb, sb = oracle.quantize(b, 1, E4M3)
    sa[1, 0] = 0xFF                      # X = NaN for one block of row 1 of A
    cb = unpack(eb, 8)
    cb[2, 40] = 0x7F                     # element NaN in row 2 of B
    eb = pack(cb, 8)
    C = oracle.gemm(ea, sa, E2M1, eb, sb, E4M3, K)
    nan = np.isnan(C)
    expect = np.zeros((4, 4), dtype=bool)
    expect[1, :] = True
    expect[:, 2] = True
    assert np.array_equal(nan, expect)


def test_rejects_bad_arguments(oracle):
    e = np.zeros((2, 48), dtype=np.uint8)
    s = np.zeros((2, 1), dtype=np.uint8)
    with pytest.raises(ValueError):
        oracle.gemm(e, s, E4M3, e, s, E4M3, 48)
    with pytest.raises(ValueError):
        oracle.gemm_entries(e, s, E4M3, e, s, E4M3, 32, [2], [0])
