"""Pins of the reference's 3-D cast (Section 3: the principal axis of a multi-dimensional
tensor).  mxo_quantize_3d walks the fibres of the tensor itself; it is held against the
2-D cast of the explicitly permuted tensor (a different routine on a different memory
order), against a by-hand block, and the source-order layout against the block-major one
re-laid out with numpy."""
import numpy as np
import pytest

from paper_2310_10537_amd import inputs

BITS = (8, 8, 6, 6, 4, 8)


def unpack(elems, w, n):
    """little-endian dense packing: bytes [..., n*w/8] -> codes [..., n]"""
    bits = np.unpackbits(elems, axis=-1, bitorder="little")[..., : n * w]
    bits = bits.reshape(elems.shape[:-1] + (n, w)).astype(np.uint32)
    return (bits << np.arange(w, dtype=np.uint32)).sum(axis=-1)


@pytest.mark.parametrize("fmt", range(6))
@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("shape", [(3, 64, 96), (5, 40, 72), (33, 2, 8)])
def test_block_major_equals_2d_cast_of_the_permuted_tensor(oracle, fmt, axis, shape):
    x = inputs.student_t_f32((shape[0] * shape[1], shape[2]), seed=7 + fmt).reshape(shape)
    for src in (x, inputs.f32_to_bf16_bits(x)):
        e, s = oracle.quantize_3d(src, axis, fmt, rnd=fmt % 2)
        moved = np.ascontiguousarray(np.moveaxis(src, axis, -1))
        e2, s2 = oracle.quantize(moved.reshape(-1, shape[axis]), 1, fmt, fmt % 2)
        assert np.array_equal(e.reshape(e2.shape), e2) and np.array_equal(s.reshape(s2.shape), s2)


@pytest.mark.parametrize("fmt", range(6))
@pytest.mark.parametrize("axis", [0, 1, 2])
def test_source_order_layout_is_the_block_major_one_re_laid_out(oracle, fmt, axis):
    shape = (40, 70, 24)        # two of the three axes end in a partial block
    w = BITS[fmt]
    x = inputs.student_t_f32((shape[0] * shape[1], shape[2]), seed=17 + fmt).reshape(shape)
    e, s = oracle.quantize_3d(x, axis, fmt)
    ek, sk = oracle.quantize_3d(x, axis, fmt, keep_order=True)
    L = shape[axis]
    nblk = -(-L // 32)
    codes = unpack(e, w, nblk * 32)[..., :L]                   # [o1][o2][L]
    codes_k = unpack(ek, w, shape[2])                          # [d0][d1][d2]
    assert np.array_equal(np.moveaxis(codes, -1, axis), codes_k)
    assert np.array_equal(np.moveaxis(s, -1, axis), sk)
    # the fill of a partial block holds code 0
    assert not unpack(e, w, nblk * 32)[..., L:].any()


def test_strides_select_a_sub_tensor(oracle):
    big = inputs.gaussian_f32((6 * 50, 80), seed=3).reshape(6, 50, 80)
    sub = big[1:5, 3:43, 16:80]
    flat = big.reshape(-1)[1 * 4000 + 3 * 80 + 16:]
    for axis in range(3):
        for keep in (False, True):
            a = oracle.quantize_3d(np.ascontiguousarray(sub), axis, 2, keep_order=keep)
            b = oracle.quantize_3d(flat, axis, 2, keep_order=keep, strides=(4000, 80, sub.shape))
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_hand_worked_fibre(oracle):
    """A [32][1][2] tensor blocked along axis 0: column 0 holds {1.0, 0.3, -0.001, 0...}
    (E4M3: scale byte 119, codes 0x78, 0x6A, 0xA8), column 1 holds 1.9 (saturates to 0x7E)."""
    x = np.zeros((32, 1, 2), np.float32)
    x[0, 0, 0], x[1, 0, 0], x[2, 0, 0] = 1.0, 0.3, -0.001
    x[5, 0, 1] = 1.9
    e, s = oracle.quantize_3d(x, 0, 0, keep_order=True)
    assert s.shape == (1, 1, 2) and s[0, 0, 0] == 119 and s[0, 0, 1] == 119
    assert e[0, 0, 0] == 0x78 and e[1, 0, 0] == 0x6A and e[2, 0, 0] == 0xA8 and e[5, 0, 1] == 0x7E
    e2, s2 = oracle.quantize_3d(x, 0, 0)
    assert e2.shape == (1, 2, 32) and e2[0, 0, 0] == 0x78 and e2[0, 1, 5] == 0x7E and s2[0, 1, 0] == 119
