"""ctypes binding of libmx.so (C ABI in include/mx.h).

Argument marshalling only: every step of the cast, the dequantize and the GEMM
runs in the HIP kernels of the library.  PyTorch is used for device memory and
for the current stream.  There is no fallback: a missing library is an error.
"""
import ctypes
import os

import torch

FP8_E4M3, FP8_E5M2, FP6_E3M2, FP6_E2M3, FP4_E2M1, INT8 = range(6)
FORMAT_NAMES = ("fp8_e4m3", "fp8_e5m2", "fp6_e3m2", "fp6_e2m3", "fp4_e2m1", "int8")
FORMAT_BITS = (8, 8, 6, 6, 4, 8)
ROUND_RNE, ROUND_HALF_AWAY, ROUND_TOWARD_ZERO, ROUND_STOCHASTIC = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1
MX_OK = 0
MX_ERR_TOO_LARGE = 7
MX_ERR_WORKSPACE = 8
NOALLOC_SCRATCH_BYTES = 36 << 20
BLOCK = 32

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmx.so")
_lib = None


class MxError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"mx status {status}: {text}")
        self.status = status


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library with argument types declared."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2310_10537_amd.build` "
                "(hipcc, --offload-arch=gfx950); there is no CPU fallback")
        L = ctypes.CDLL(_LIB_PATH)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.mx_elem_bytes.argtypes = [ci, i64, i64, ci]
        L.mx_elem_bytes.restype = ctypes.c_size_t
        L.mx_scale_bytes.argtypes = [i64, i64, ci]
        L.mx_scale_bytes.restype = ctypes.c_size_t
        L.mx_quantize.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, vp, vp, vp]
        L.mx_quantize_sr.argtypes = [vp, ci, i64, i64, i64, ci, ci, ctypes.c_uint64, vp, vp, vp]
        L.mx_quantize_dual.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, vp, vp, vp, vp]
        L.mx_dequantize.argtypes = [vp, vp, ci, i64, i64, ci, vp, ci, i64, vp]
        L.mx_gemm.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, vp, ci, i64, vp]
        L.mx_gemm_qa.argtypes = [i64, i64, i64, vp, i64, ci, ci, vp, vp, ci, vp, ci, i64, vp]
        L.mx_gemm_q.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, ci, ci, vp, vp, vp]
        L.mx_gemm_qa_noalloc.argtypes = [i64, i64, i64, vp, i64, ci, ci, vp, vp, ci, vp, ci, i64, vp]
        sz = ctypes.c_size_t
        for name in ("mx_gemm_workspace_bytes", "mx_gemm_qa_workspace_bytes", "mx_gemm_q_workspace_bytes"):
            getattr(L, name).argtypes = [i64, i64, i64, ci, ci]
            getattr(L, name).restype = sz
        L.mx_gemm_ws.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, vp, ci, i64, vp, sz, vp]
        L.mx_gemm_qa_ws.argtypes = [i64, i64, i64, vp, i64, ci, ci, vp, vp, ci, vp, ci, i64, vp, sz, vp]
        L.mx_gemm_q_ws.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, ci, ci, vp, vp, vp, sz, vp]
        L.mx_dequantize_3d.argtypes = [vp, vp, ci, i64, i64, i64, ci, ci, vp, ci, i64, i64, vp]
        L.mx_quantize_3d.argtypes = [vp, ci, i64, i64, i64, i64, i64, ci, ci, ci, ci, vp, vp, vp]
        L.mx_stream_pattern.argtypes = [vp, vp, i64, ci, ci, vp]
        L.mx_gemm_probe.argtypes = [i64, i64, i64, vp, vp, ci, vp, vp, ci, vp, i64, vp, i64, vp]
        L.mx_mfma_stream_probe.argtypes = [ci, vp, ci, vp, vp, vp]
        L.mx_strerror.argtypes = [ci]
        L.mx_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(status: int):
    if status != MX_OK:
        raise MxError(status, lib().mx_strerror(status).decode())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DT_F32
    if t.dtype == torch.bfloat16:
        return DT_BF16
    raise TypeError("tensor must be float32 or bfloat16")


def _dev(t: torch.Tensor, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")


def mx_elem_bytes(fmt, rows, cols, axis=1):
    return lib().mx_elem_bytes(fmt, rows, cols, axis)


def mx_scale_bytes(rows, cols, axis=1):
    return lib().mx_scale_bytes(rows, cols, axis)


def mx_strerror(status):
    return lib().mx_strerror(status).decode()


def mx_quantize(src, axis, fmt, rnd=ROUND_RNE, elems_out=None, scales_out=None, stream=None):
    """src: 2-D device tensor (float32 / bfloat16, last dim contiguous).
    Returns (elems uint8 [n_out, len*bits/8], scales uint8 [n_out, len/32])."""
    _dev(src, "src")
    assert src.dim() == 2 and (src.shape[1] == 0 or src.stride(1) == 1)
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else cols
    n_out, length = (rows, cols) if axis == 1 else (cols, rows)
    w = FORMAT_BITS[fmt] if 0 <= fmt < 6 else 8
    nblk = -(-length // BLOCK)      # a partial last block is stored whole
    if elems_out is None:
        elems_out = torch.empty((n_out, nblk * BLOCK * w // 8), dtype=torch.uint8, device=src.device)
    if scales_out is None:
        scales_out = torch.empty((n_out, nblk), dtype=torch.uint8, device=src.device)
    _check(lib().mx_quantize(src.data_ptr(), _dt(src), rows, cols, ld, axis, fmt, rnd,
                             elems_out.data_ptr(), scales_out.data_ptr(), _stream(stream)))
    return elems_out, scales_out


def mx_quantize_sr(src, axis, fmt, seed, elems_out=None, scales_out=None, stream=None):
    """mx_quantize with stochastic rounding; the random offset of an element is a function of
    (seed, its index in src) only."""
    _dev(src, "src")
    assert src.dim() == 2 and (src.shape[1] == 0 or src.stride(1) == 1)
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else cols
    n_out, length = (rows, cols) if axis == 1 else (cols, rows)
    w = FORMAT_BITS[fmt] if 0 <= fmt < 6 else 8
    nblk = -(-length // BLOCK)      # a partial last block is stored whole
    if elems_out is None:
        elems_out = torch.empty((n_out, nblk * BLOCK * w // 8), dtype=torch.uint8, device=src.device)
    if scales_out is None:
        scales_out = torch.empty((n_out, nblk), dtype=torch.uint8, device=src.device)
    _check(lib().mx_quantize_sr(src.data_ptr(), _dt(src), rows, cols, ld, axis, fmt, int(seed) & (2 ** 64 - 1),
                                elems_out.data_ptr(), scales_out.data_ptr(), _stream(stream)))
    return elems_out, scales_out


def mx_quantize_dual(src, fmt, rnd=ROUND_RNE, out_axis1=None, out_axis0=None, stream=None):
    """Both casts of src in one call.  Returns ((elems, scales) for axis 1, (elems, scales) for axis 0)."""
    _dev(src, "src")
    assert src.dim() == 2 and (src.shape[1] == 0 or src.stride(1) == 1)
    rows, cols = src.shape
    ld = src.stride(0) if rows > 1 else cols
    w = FORMAT_BITS[fmt] if 0 <= fmt < 6 else 8
    if out_axis1 is None:
        out_axis1 = (torch.empty((rows, cols * w // 8), dtype=torch.uint8, device=src.device),
                     torch.empty((rows, cols // BLOCK), dtype=torch.uint8, device=src.device))
    if out_axis0 is None:
        out_axis0 = (torch.empty((cols, rows * w // 8), dtype=torch.uint8, device=src.device),
                     torch.empty((cols, rows // BLOCK), dtype=torch.uint8, device=src.device))
    _check(lib().mx_quantize_dual(src.data_ptr(), _dt(src), rows, cols, ld, fmt, rnd,
                                  out_axis1[0].data_ptr(), out_axis1[1].data_ptr(),
                                  out_axis0[0].data_ptr(), out_axis0[1].data_ptr(), _stream(stream)))
    return out_axis1, out_axis0


def mx_dequantize(elems, scales, fmt, rows, cols, axis, dtype=torch.float32, out=None, stream=None):
    """Returns the row-major [rows, cols] tensor of X * P."""
    _dev(elems, "elems")
    _dev(scales, "scales")
    if out is None:
        out = torch.empty((rows, cols), dtype=dtype, device=elems.device)
    ld = out.stride(0) if rows > 1 else cols
    _check(lib().mx_dequantize(elems.data_ptr(), scales.data_ptr(), fmt, rows, cols, axis,
                               out.data_ptr(), _dt(out), ld, _stream(stream)))
    return out


def mx_gemm(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, dtype=torch.float32, out=None, stream=None):
    """C[M, N] = A[M, K] . B[N, K]^T on MX operands blocked along K."""
    for t, n in ((A_elems, "A_elems"), (A_scales, "A_scales"), (B_elems, "B_elems"), (B_scales, "B_scales")):
        _dev(t, n)
    M, N = A_scales.shape[0], B_scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=A_elems.device)
    ldc = out.stride(0) if M > 1 else N
    _check(lib().mx_gemm(M, N, K, A_elems.data_ptr(), A_scales.data_ptr(), fmtA,
                         B_elems.data_ptr(), B_scales.data_ptr(), fmtB,
                         out.data_ptr(), _dt(out), ldc, _stream(stream)))
    return out


def mx_gemm_q(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, fmtC, rnd=ROUND_RNE, out=None, stream=None):
    """C = A . B^T delivered as an MX tensor blocked along N.  Returns (elems, scales)."""
    for t, n in ((A_elems, "A_elems"), (A_scales, "A_scales"), (B_elems, "B_elems"), (B_scales, "B_scales")):
        _dev(t, n)
    M, N = A_scales.shape[0], B_scales.shape[0]
    w = FORMAT_BITS[fmtC] if 0 <= fmtC < 6 else 8
    nblk = -(-N // BLOCK)
    if out is None:
        out = (torch.empty((M, nblk * BLOCK * w // 8), dtype=torch.uint8, device=A_elems.device),
               torch.empty((M, nblk), dtype=torch.uint8, device=A_elems.device))
    _check(lib().mx_gemm_q(M, N, K, A_elems.data_ptr(), A_scales.data_ptr(), fmtA, B_elems.data_ptr(), B_scales.data_ptr(),
                           fmtB, fmtC, rnd, out[0].data_ptr(), out[1].data_ptr(), _stream(stream)))
    return out


def mx_gemm_qa(A_bf16, fmtA, rnd, B_elems, B_scales, fmtB, dtype=torch.float32, out=None, stream=None):
    """Same product with A given as raw bf16 [M, K] and cast to fmtA on load."""
    _dev(A_bf16, "A_bf16")
    _dev(B_elems, "B_elems")
    _dev(B_scales, "B_scales")
    assert A_bf16.dtype == torch.bfloat16 and A_bf16.dim() == 2
    M, K = A_bf16.shape
    N = B_scales.shape[0]
    lda = A_bf16.stride(0) if M > 1 else K
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=A_bf16.device)
    ldc = out.stride(0) if M > 1 else N
    _check(lib().mx_gemm_qa(M, N, K, A_bf16.data_ptr(), lda, fmtA, rnd,
                            B_elems.data_ptr(), B_scales.data_ptr(), fmtB,
                            out.data_ptr(), _dt(out), ldc, _stream(stream)))
    return out


def mx_gemm_qa_noalloc(A_bf16, fmtA, rnd, B_elems, B_scales, fmtB, out, stream=None):
    """mx_gemm_qa without any device allocation by the library: the MX form of A lives in the
    library's static scratch array (NOALLOC_SCRATCH_BYTES).  `out` is required: this wrapper
    allocates nothing either."""
    _dev(A_bf16, "A_bf16")
    _dev(B_elems, "B_elems")
    _dev(B_scales, "B_scales")
    _dev(out, "out")
    assert A_bf16.dtype == torch.bfloat16 and A_bf16.dim() == 2
    M, K = A_bf16.shape
    N = B_scales.shape[0]
    lda = A_bf16.stride(0) if M > 1 else K
    ldc = out.stride(0) if M > 1 else N
    _check(lib().mx_gemm_qa_noalloc(M, N, K, A_bf16.data_ptr(), lda, fmtA, rnd,
                                    B_elems.data_ptr(), B_scales.data_ptr(), fmtB,
                                    out.data_ptr(), _dt(out), ldc, _stream(stream)))
    return out


def mx_stream_pattern(src, dst, dst_bytes, read_per_write, write, stream=None):
    """Measurement aid: read read_per_write * dst_bytes from src, write dst_bytes to dst (if write)."""
    _check(lib().mx_stream_pattern(src.data_ptr() if src is not None else None, dst.data_ptr(), dst_bytes,
                                   read_per_write, 1 if write else 0, _stream(stream)))


def mx_quantize_3d(src, axis, fmt, rnd=ROUND_RNE, keep_order=False, stream=None):
    """src: 3-D device tensor (float32 / bfloat16), last dim contiguous, any strides on the first two.
    Returns (elems, scales) in the layout mx_quantize_3d documents."""
    _dev(src, "src")
    assert src.dim() == 3 and (src.shape[2] == 0 or src.stride(2) == 1)
    d0, d1, d2 = src.shape
    s1 = src.stride(1) if d1 > 1 else d2
    s0 = src.stride(0) if d0 > 1 else d1 * s1
    w = FORMAT_BITS[fmt] if 0 <= fmt < 6 else 8
    dim = (d0, d1, d2)
    nblk = -(-dim[axis] // BLOCK) if 0 <= axis < 3 else 1
    if keep_order:
        elems = torch.empty((d0, d1, d2 * w // 8), dtype=torch.uint8, device=src.device)
        sshape = list(dim)
        if 0 <= axis < 3:
            sshape[axis] = nblk
        scales = torch.empty(sshape, dtype=torch.uint8, device=src.device)
    else:
        rest = [dim[i] for i in range(3) if i != axis][:2] if 0 <= axis < 3 else [d0, d1]
        elems = torch.empty((rest[0], rest[1], nblk * BLOCK * w // 8), dtype=torch.uint8, device=src.device)
        scales = torch.empty((rest[0], rest[1], nblk), dtype=torch.uint8, device=src.device)
    _check(lib().mx_quantize_3d(src.data_ptr(), _dt(src), d0, d1, d2, s0, s1, axis, fmt, rnd, 1 if keep_order else 0,
                                elems.data_ptr(), scales.data_ptr(), _stream(stream)))
    return elems, scales


def _ws_args(workspace):
    if workspace is None:
        return None, 0
    _dev(workspace, "workspace")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def mx_gemm_ws(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, workspace, dtype=torch.float32, out=None, stream=None):
    """mx_gemm with the scratch memory (if the route needs any) taken from `workspace`, a device tensor of at
    least mx_gemm_workspace_bytes(...) bytes."""
    M, N = A_scales.shape[0], B_scales.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=A_elems.device)
    ldc = out.stride(0) if M > 1 else N
    wp, wb = _ws_args(workspace)
    _check(lib().mx_gemm_ws(M, N, K, A_elems.data_ptr(), A_scales.data_ptr(), fmtA, B_elems.data_ptr(), B_scales.data_ptr(), fmtB,
                            out.data_ptr(), _dt(out), ldc, wp, wb, _stream(stream)))
    return out


def mx_gemm_qa_ws(A_bf16, fmtA, rnd, B_elems, B_scales, fmtB, workspace, dtype=torch.float32, out=None, stream=None):
    M, K = A_bf16.shape
    N = B_scales.shape[0]
    lda = A_bf16.stride(0) if M > 1 else K
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=A_bf16.device)
    ldc = out.stride(0) if M > 1 else N
    wp, wb = _ws_args(workspace)
    _check(lib().mx_gemm_qa_ws(M, N, K, A_bf16.data_ptr(), lda, fmtA, rnd, B_elems.data_ptr(), B_scales.data_ptr(), fmtB,
                               out.data_ptr(), _dt(out), ldc, wp, wb, _stream(stream)))
    return out


def mx_gemm_q_ws(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, fmtC, rnd, workspace, out=None, stream=None):
    M, N = A_scales.shape[0], B_scales.shape[0]
    w = FORMAT_BITS[fmtC] if 0 <= fmtC < 6 else 8
    nblk = -(-N // BLOCK)
    if out is None:
        out = (torch.empty((M, nblk * BLOCK * w // 8), dtype=torch.uint8, device=A_elems.device),
               torch.empty((M, nblk), dtype=torch.uint8, device=A_elems.device))
    wp, wb = _ws_args(workspace)
    _check(lib().mx_gemm_q_ws(M, N, K, A_elems.data_ptr(), A_scales.data_ptr(), fmtA, B_elems.data_ptr(), B_scales.data_ptr(),
                              fmtB, fmtC, rnd, out[0].data_ptr(), out[1].data_ptr(), wp, wb, _stream(stream)))
    return out


def mx_workspace_bytes(kind, M, N, K, fmtA, fmtB):
    """kind: "gemm", "gemm_qa" or "gemm_q"."""
    return getattr(lib(), f"mx_{kind}_workspace_bytes")(M, N, K, fmtA, fmtB)


def mx_gemm_probe(A_elems, A_scales, fmtA, B_elems, B_scales, fmtB, K, out, stream=None):
    """Measurement aid: the tiled GEMM with per-work-group timing.  Returns (shader clocks, 100 MHz ticks)
    of the work-groups' K loops as two int64 tensors (work-groups that had a tile only)."""
    M, N = A_scales.shape[0], B_scales.shape[0]
    wgs = (-(-((M // 256) * (N // 256)) // 8)) * 8
    probe = torch.zeros((wgs, 2), dtype=torch.int64, device=A_elems.device)
    _check(lib().mx_gemm_probe(M, N, K, A_elems.data_ptr(), A_scales.data_ptr(), fmtA, B_elems.data_ptr(), B_scales.data_ptr(), fmtB,
                               out.data_ptr(), out.stride(0), probe.data_ptr(), probe.numel(), _stream(stream)))
    ran = probe[:, 1] > 0
    return probe[ran, 0], probe[ran, 1]


MX_MFMA_STREAM_WGS = 256


def mx_mfma_stream_probe(fmt, codes, iters, stream=None):
    """Measurement aid: the GEMM kernels' matrix instruction alone, from registers filled with the first 64 KiB
    of `codes` (uint8, device).  Returns (shader clocks, 100 MHz ticks) per work-group as two int64 tensors;
    one launch performs MX_MFMA_STREAM_WGS * 4 * 16 * iters * 131072 flops."""
    _dev(codes, "codes")
    assert codes.dtype == torch.uint8 and codes.is_contiguous() and codes.numel() >= 65536
    probe = torch.zeros((MX_MFMA_STREAM_WGS, 2), dtype=torch.int64, device=codes.device)
    sink = torch.empty((MX_MFMA_STREAM_WGS * 256,), dtype=torch.float32, device=codes.device)
    _check(lib().mx_mfma_stream_probe(fmt, codes.data_ptr(), iters, sink.data_ptr(), probe.data_ptr(), _stream(stream)))
    return probe[:, 0], probe[:, 1]


def mx_dequantize_3d(elems, scales, fmt, shape, axis, keep_order=False, dtype=torch.float32, out=None, stream=None):
    """Inverse of mx_quantize_3d.  out: a [d0, d1, d2] tensor whose last axis is contiguous (strides are taken
    from it); a dense one is allocated when it is None."""
    _dev(elems, "elems")
    _dev(scales, "scales")
    d0, d1, d2 = shape
    if out is None:
        out = torch.empty((d0, d1, d2), dtype=dtype, device=elems.device)
    assert tuple(out.shape) == (d0, d1, d2) and (d2 == 0 or out.stride(2) == 1)
    s0 = out.stride(0) if d0 > 1 else d1 * max(out.stride(1), d2)
    s1 = out.stride(1) if d1 > 1 else d2
    _check(lib().mx_dequantize_3d(elems.data_ptr(), scales.data_ptr(), fmt, d0, d1, d2, axis, 1 if keep_order else 0,
                                  out.data_ptr(), _dt(out), s0, s1, _stream(stream)))
    return out
