"""Reference CPU implementation of the MX cast / dequantize / dot product.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg; never by the GPU package.  Thin ctypes layer
over oracle/libmx_oracle.so (plain C, see mx_oracle.c); all arrays are numpy
arrays in host memory.
"""
import ctypes
import os

import numpy as np

FP8_E4M3, FP8_E5M2, FP6_E3M2, FP6_E2M3, FP4_E2M1, INT8 = range(6)
FORMATS = (FP8_E4M3, FP8_E5M2, FP6_E3M2, FP6_E2M3, FP4_E2M1, INT8)
FORMAT_NAMES = ("fp8_e4m3", "fp8_e5m2", "fp6_e3m2", "fp6_e2m3", "fp4_e2m1", "int8")
ROUND_RNE, ROUND_HALF_AWAY, ROUND_TOWARD_ZERO, ROUND_STOCHASTIC = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1
BLOCK = 32

_lib = None


def lib():
    global _lib
    if _lib is None:
        from . import build as _build
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.mxo_elem_bits.argtypes = [ci]
        L.mxo_emax.argtypes = [ci]
        L.mxo_decode.argtypes = [ci, ctypes.c_uint]
        L.mxo_decode.restype = ctypes.c_double
        L.mxo_encode.argtypes = [ci, ci, ctypes.c_double]
        L.mxo_encode.restype = ctypes.c_uint
        L.mxo_quantize_block.argtypes = [vp, ci, ci, vp, vp]
        L.mxo_quantize_block.restype = None
        L.mxo_quantize.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, vp, vp]
        L.mxo_quantize_seeded.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, ctypes.c_uint64, vp, vp]
        L.mxo_encode_u.argtypes = [ci, ci, ctypes.c_double, ctypes.c_double]
        L.mxo_encode_u.restype = ctypes.c_uint
        L.mxo_quantize_block_u.argtypes = [vp, ci, ci, vp, vp, vp]
        L.mxo_quantize_block_u.restype = None
        L.mxo_philox4x32.argtypes = [ctypes.c_uint64, ctypes.c_uint64, vp]
        L.mxo_philox4x32.restype = None
        L.mxo_philox4x32_words.argtypes = [vp, vp, vp]
        L.mxo_philox4x32_words.restype = None
        L.mxo_sr_uniform.argtypes = [ctypes.c_uint64, i64]
        L.mxo_sr_uniform.restype = ctypes.c_double
        L.mxo_quantize_3d.argtypes = [vp, ci, i64, i64, i64, i64, i64, ci, ci, ci, ci, vp, vp]
        L.mxo_dequantize.argtypes = [vp, vp, ci, i64, i64, ci, vp, ci, i64]
        L.mxo_dequantize_3d.argtypes = [vp, vp, ci, i64, i64, i64, ci, ci, vp, ci, i64, i64]
        L.mxo_gemm.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, vp, vp]
        L.mxo_gemm_entries.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, i64, vp, vp, vp, vp]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def elem_bits(fmt):
    return lib().mxo_elem_bits(fmt)


def emax(fmt):
    return lib().mxo_emax(fmt)


def decode(fmt, code):
    return lib().mxo_decode(fmt, int(code))


def encode(fmt, rnd, x, u=0.0):
    return lib().mxo_encode_u(fmt, rnd, float(x), float(u))


def philox4x32(key, counter):
    """Philox4x32-10 with a 64-bit key and a 64-bit counter (upper counter words 0)."""
    out = np.zeros(4, dtype=np.uint32)
    lib().mxo_philox4x32(int(key), int(counter), _ptr(out))
    return out


def philox4x32_words(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().mxo_philox4x32_words(_ptr(c), _ptr(k), _ptr(out))
    return out


def sr_uniform(seed, e):
    return lib().mxo_sr_uniform(int(seed), int(e))


def num_threads():
    return lib().mxo_num_threads()


def quantize_block(values, fmt, rnd=ROUND_RNE, u=None):
    """values: 32 floats (widened to double); u: 32 random offsets in [0, 1) for the
    stochastic mode.  Returns (scale_byte, codes[32])."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    assert v.shape == (BLOCK,)
    scale = np.zeros(1, dtype=np.uint8)
    codes = np.zeros(BLOCK, dtype=np.uint32)
    if u is None:
        lib().mxo_quantize_block(_ptr(v), fmt, rnd, _ptr(scale), _ptr(codes))
    else:
        uu = np.ascontiguousarray(u, dtype=np.float64)
        assert uu.shape == (BLOCK,)
        lib().mxo_quantize_block_u(_ptr(v), fmt, rnd, _ptr(uu), _ptr(scale), _ptr(codes))
    return int(scale[0]), codes


def _src_dt(src):
    """src is float32, or uint16 holding bf16 bit patterns."""
    if src.dtype == np.float32:
        return DT_F32
    if src.dtype == np.uint16:
        return DT_BF16
    raise TypeError("source must be float32 or uint16 (bf16 bits)")


def quantize(src, axis, fmt, rnd=ROUND_RNE, seed=None):
    """src: 2-D C-contiguous float32 array or uint16 array of bf16 bits.
    seed: required by (and only by) the stochastic mode.
    Returns (elems uint8 [n_out, len*bits/8], scales uint8 [n_out, len/32])."""
    src = np.ascontiguousarray(src)
    rows, cols = src.shape
    n_out, length = (rows, cols) if axis == 1 else (cols, rows)
    w = elem_bits(fmt)
    nblk = -(-length // BLOCK)          # a partial last block is stored whole (zero fill)
    elems = np.zeros((n_out, nblk * BLOCK * w // 8), dtype=np.uint8)
    scales = np.zeros((n_out, nblk), dtype=np.uint8)
    if (rnd == ROUND_STOCHASTIC) != (seed is not None):
        raise ValueError("a seed goes with the stochastic mode and with no other")
    st = lib().mxo_quantize_seeded(_ptr(src), _src_dt(src), rows, cols, cols, axis, fmt, rnd,
                                   int(seed or 0), _ptr(elems), _ptr(scales))
    if st != 0:
        raise ValueError("mxo_quantize rejected its arguments")
    return elems, scales


def quantize_3d(src, axis, fmt, rnd=ROUND_RNE, keep_order=False, strides=None):
    """src: 3-D float32 array or uint16 array of bf16 bits; strides (stride0, stride1) in elements
    when src is a flat buffer holding a strided tensor of shape `strides[2:]` (else C-contiguous).
    Returns (elems, scales) shaped as mxo_quantize_3d documents."""
    if strides is None:
        src = np.ascontiguousarray(src)
        d0, d1, d2 = src.shape
        s0, s1 = d1 * d2, d2
    else:
        s0, s1, (d0, d1, d2) = strides[0], strides[1], strides[2]
        src = np.ascontiguousarray(src).reshape(-1)
        assert (d0 - 1) * s0 + (d1 - 1) * s1 + d2 <= src.size
    w = elem_bits(fmt)
    dim = (d0, d1, d2)
    nblk = -(-dim[axis] // BLOCK)
    if keep_order:
        elems = np.zeros((d0, d1, d2 * w // 8), dtype=np.uint8)
        sshape = list(dim)
        sshape[axis] = nblk
        scales = np.zeros(sshape, dtype=np.uint8)
    else:
        rest = [dim[i] for i in range(3) if i != axis]
        elems = np.zeros((rest[0], rest[1], nblk * BLOCK * w // 8), dtype=np.uint8)
        scales = np.zeros((rest[0], rest[1], nblk), dtype=np.uint8)
    st = lib().mxo_quantize_3d(_ptr(src), _src_dt(src), d0, d1, d2, s0, s1, axis, fmt, rnd, 1 if keep_order else 0,
                               _ptr(elems), _ptr(scales))
    if st != 0:
        raise ValueError("mxo_quantize_3d rejected its arguments")
    return elems, scales


def dequantize_3d(elems, scales, fmt, shape, axis, keep_order=False, dst_dt=DT_F32, strides=None):
    """Inverse of quantize_3d.  Returns the [d0, d1, d2] tensor (float32, or uint16 bf16 bits); with
    strides = (stride0, stride1) a flat buffer of (d0 - 1) * stride0 + (d1 - 1) * stride1 + d2 entries
    whose untouched entries keep the value 0x7777 / 7.0 (so a test sees what was written)."""
    d0, d1, d2 = shape
    elems = np.ascontiguousarray(elems, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    dt = np.float32 if dst_dt == DT_F32 else np.uint16
    if strides is None:
        dst = np.zeros((d0, d1, d2), dtype=dt)
        s0, s1 = d1 * d2, d2
    else:
        s0, s1 = strides
        dst = np.full((d0 - 1) * s0 + (d1 - 1) * s1 + d2, 7.0 if dst_dt == DT_F32 else 0x7777, dtype=dt)
    st = lib().mxo_dequantize_3d(_ptr(elems), _ptr(scales), fmt, d0, d1, d2, axis, 1 if keep_order else 0, _ptr(dst), dst_dt, s0, s1)
    if st != 0:
        raise ValueError("mxo_dequantize_3d rejected its arguments")
    return dst


def dequantize(elems, scales, fmt, rows, cols, axis, dst_dt=DT_F32):
    """Returns float32 [rows, cols], or uint16 bf16 bits when dst_dt is DT_BF16."""
    elems = np.ascontiguousarray(elems, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    dst = np.zeros((rows, cols), dtype=np.float32 if dst_dt == DT_F32 else np.uint16)
    st = lib().mxo_dequantize(_ptr(elems), _ptr(scales), fmt, rows, cols, axis,
                              _ptr(dst), dst_dt, cols)
    if st != 0:
        raise ValueError("mxo_dequantize rejected its arguments")
    return dst


def gemm(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, want_abs=False):
    """C[M,N] (float64) = A[M,K] . B[N,K]^T on MX operands blocked along K."""
    A_elems = np.ascontiguousarray(A_elems, dtype=np.uint8)
    B_elems = np.ascontiguousarray(B_elems, dtype=np.uint8)
    A_scales = np.ascontiguousarray(A_scales, dtype=np.uint8)
    B_scales = np.ascontiguousarray(B_scales, dtype=np.uint8)
    M, N = A_scales.shape[0], B_scales.shape[0]
    C = np.zeros((M, N), dtype=np.float64)
    Cabs = np.zeros((M, N), dtype=np.float64) if want_abs else None
    st = lib().mxo_gemm(M, N, K, _ptr(A_elems), _ptr(A_scales), fmtA,
                        _ptr(B_elems), _ptr(B_scales), fmtB, _ptr(C),
                        _ptr(Cabs) if want_abs else None)
    if st != 0:
        raise ValueError("mxo_gemm rejected its arguments")
    return (C, Cabs) if want_abs else C


def gemm_entries(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, mi, ni):
    """Dot products for the listed (m, n) pairs.  Returns (C, Cabs) float64 [n]."""
    A_elems = np.ascontiguousarray(A_elems, dtype=np.uint8)
    B_elems = np.ascontiguousarray(B_elems, dtype=np.uint8)
    A_scales = np.ascontiguousarray(A_scales, dtype=np.uint8)
    B_scales = np.ascontiguousarray(B_scales, dtype=np.uint8)
    mi = np.ascontiguousarray(mi, dtype=np.int64)
    ni = np.ascontiguousarray(ni, dtype=np.int64)
    M, N = A_scales.shape[0], B_scales.shape[0]
    C = np.zeros(mi.shape[0], dtype=np.float64)
    Cabs = np.zeros(mi.shape[0], dtype=np.float64)
    st = lib().mxo_gemm_entries(M, N, K, _ptr(A_elems), _ptr(A_scales), fmtA,
                                _ptr(B_elems), _ptr(B_scales), fmtB, mi.shape[0],
                                _ptr(mi), _ptr(ni), _ptr(C), _ptr(Cabs))
    if st != 0:
        raise ValueError("mxo_gemm_entries rejected its arguments")
    return C, Cabs
