"""The C-ABI library loads and exports every symbol include/mx.h declares, and
its argument validation (which runs before any HIP call) returns the documented
status codes.  No GPU needed: nothing here launches a kernel."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2310_10537_amd import binding
    if not os.path.exists(binding._LIB_PATH):
        from paper_2310_10537_amd import build
        build.build()
    return binding.lib()


def test_exports_match_header(L):
    text = open(os.path.join(ROOT, "include", "mx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(mx_[a-z0-9_]+)\s*\(", text))
    assert names == {"mx_elem_bytes", "mx_scale_bytes", "mx_quantize", "mx_quantize_sr", "mx_quantize_dual", "mx_quantize_3d", "mx_dequantize", "mx_gemm",
                     "mx_gemm_qa", "mx_gemm_q", "mx_gemm_qa_noalloc", "mx_stream_pattern", "mx_strerror",
                     "mx_gemm_workspace_bytes", "mx_gemm_qa_workspace_bytes", "mx_gemm_q_workspace_bytes", "mx_gemm_ws", "mx_gemm_qa_ws",
                     "mx_gemm_q_ws", "mx_gemm_probe", "mx_mfma_stream_probe", "mx_dequantize_3d"}
    for n in names:
        assert hasattr(L, n), n


def test_sizes(L):
    assert L.mx_elem_bytes(0, 1024, 1024, 1) == 1024 * 1024
    assert L.mx_elem_bytes(2, 64, 64, 0) == 64 * 64 * 6 // 8
    assert L.mx_elem_bytes(4, 8192, 8192, 1) == 8192 * 8192 // 2
    assert L.mx_scale_bytes(8192, 8192, 0) == 8192 * 8192 // 32
    assert L.mx_elem_bytes(9, 4, 32, 1) == 0
    # a partial last block is stored whole
    assert L.mx_elem_bytes(2, 10, 33, 1) == 10 * 2 * 24 and L.mx_scale_bytes(10, 33, 1) == 20
    assert L.mx_elem_bytes(4, 33, 10, 0) == 10 * 2 * 16 and L.mx_scale_bytes(33, 10, 0) == 20
    assert L.mx_elem_bytes(0, 33, 10, 1) == 33 * 32 and L.mx_scale_bytes(33, 10, 1) == 33


def test_status_codes(L):
    OK, NULL, ENUM, SHAPE, ALIGN, UNSUP = 0, 1, 2, 3, 4, 5
    p = 0x1000  # an aligned non-null address; validation fails before it is ever used
    q = L.mx_quantize
    assert q(None, 1, 32, 32, 32, 1, 0, 0, p, p, None) == NULL
    assert q(p, 1, 32, 32, 32, 1, 6, 0, p, p, None) == ENUM
    assert q(p, 2, 32, 32, 32, 1, 0, 0, p, p, None) == ENUM
    assert q(p, 1, 32, 32, 32, 1, 0, 3, p, p, None) == ENUM      # stochastic rounding needs a seed: mx_quantize_sr
    assert q(p, 1, 32, 32, 32, 1, 0, 4, p, p, None) == ENUM
    assert q(None, 1, 32, 32, 32, 1, 0, 2, p, p, None) == NULL   # toward zero is a mode of mx_quantize
    assert q(p, 1, 32, 32, 32, 2, 0, 0, p, p, None) == ENUM
    assert q(p, 1, -1, 32, 32, 1, 0, 0, p, p, None) == SHAPE
    assert q(p, 1, 32, 64, 32, 1, 0, 0, p, p, None) == SHAPE     # ld < cols
    assert q(p + 2, 1, 32, 32, 32, 1, 0, 0, p, p, None) == ALIGN
    assert q(p, 1, 32, 32, 36, 1, 0, 0, p, p, None) == ALIGN     # 36 bf16 = 72 bytes per row
    assert q(p, 1, 32, 32, 32, 1, 0, 0, p, p + 8, None) == ALIGN
    assert q(None, 1, 0, 32, 32, 1, 0, 0, None, None, None) == OK  # empty: nothing to do
    assert q(None, 1, 32, 0, 0, 0, 0, 0, None, None, None) == OK
    qs = L.mx_quantize_sr
    assert qs(None, 1, 32, 32, 32, 1, 0, 7, p, p, None) == NULL
    assert qs(p, 1, 32, 32, 32, 1, 6, 7, p, p, None) == ENUM
    assert qs(p, 1, 32, 48, 40, 1, 0, 7, p, p, None) == SHAPE     # ld < cols
    assert qs(p, 1, 32, 32, 32, 1, 0, 7, p + 4, p, None) == ALIGN
    assert qs(None, 1, 0, 32, 32, 1, 0, 7, None, None, None) == OK
    qd = L.mx_quantize_dual
    assert qd(p, 1, 32, 32, 32, 0, 3, p, p, p, p, None) == ENUM
    assert qd(p, 1, 32, 32, 32, 0, 0, p, p, p, None, None) == NULL
    assert qd(p, 1, 32, 32, 32, 6, 0, p, p, p, p, None) == ENUM
    assert qd(p, 1, 48, 32, 32, 0, 0, p, p, p, p, None) == SHAPE    # both axes must be multiples of 32
    assert qd(p, 1, 32, 48, 48, 0, 0, p, p, p, p, None) == SHAPE
    assert qd(p, 1, 32, 32, 32, 0, 0, p, p, p + 4, p, None) == ALIGN
    assert qd(None, 1, 0, 32, 32, 0, 0, None, None, None, None, None) == OK
    d = L.mx_dequantize
    assert d(p, None, 0, 32, 32, 1, p, 0, 32, None) == NULL
    assert d(p, p, 0, 32, 40, 1, p, 0, 32, None) == SHAPE        # ld < cols
    assert d(p, p, 7, 32, 32, 1, p, 0, 32, None) == ENUM
    assert d(p, p, 0, 32, 32, 1, p + 4, 0, 32, None) == ALIGN
    g = L.mx_gemm
    assert g(16, 16, 32, p, p, 0, p, p, 0, None, 0, 16, None) == NULL
    assert g(16, 16, 48, p, p, 0, p, p, 0, p, 0, 16, None) == SHAPE
    assert g(16, 16, 32, p, p, 0, p, p, 0, p, 0, 8, None) == SHAPE   # ldc < N
    assert g(16, 16, 32, p, p, 5, p, p, 0, p, 0, 16, None) == UNSUP  # MXINT8 operand
    assert g(16, 16, 32, p, p, 0, p, p, 5, p, 0, 16, None) == UNSUP
    assert g(16, 16, 32, p, p, 5, p, p, 5, None, 0, 16, None) == NULL   # MXINT8 pairs with MXINT8
    assert g(16, 16, 32, p, p, 0, p, p, 0, p + 4, 1, 16, None) == ALIGN
    assert g(0, 16, 32, None, None, 0, None, None, 0, None, 0, 16, None) == OK
    ga = L.mx_gemm_qa
    assert ga(16, 16, 32, None, 32, 0, 0, p, p, 0, p, 0, 16, None) == NULL
    assert ga(16, 16, 32, p, 16, 0, 0, p, p, 0, p, 0, 16, None) == SHAPE  # lda < K
    assert ga(16, 16, 32, p, 36, 0, 0, p, p, 0, p, 0, 16, None) == ALIGN
    assert ga(16, 16, 32, p, 32, 0, 3, p, p, 0, p, 0, 16, None) == ENUM
    gq = L.mx_gemm_q
    assert gq(16, 32, 32, p, p, 0, p, p, 0, 0, 0, None, p, None) == NULL
    assert gq(16, 32, 32, p, p, 0, p, p, 0, 6, 0, p, p, None) == ENUM
    assert gq(16, 32, 32, p, p, 0, p, p, 0, 0, 3, p, p, None) == ENUM      # no seed here: stochastic is refused
    assert gq(16, 32, 48, p, p, 0, p, p, 0, 0, 0, p, p, None) == SHAPE
    assert gq(16, 32, 32, p, p, 5, p, p, 0, 0, 0, p, p, None) == UNSUP
    assert gq(16, 32, 32, p, p, 0, p, p, 0, 0, 0, p + 8, p, None) == ALIGN
    assert gq(0, 32, 32, None, None, 0, None, None, 0, 0, 0, None, None, None) == OK
    for s in range(8):
        assert isinstance(L.mx_strerror(s), bytes) and L.mx_strerror(s)


def test_binding_refuses_host_tensors():
    import torch
    from paper_2310_10537_amd import binding
    with pytest.raises(ValueError):
        binding.mx_quantize(torch.zeros(32, 32), 1, 0)


def test_noalloc_entry_point_validation(L):
    """mx_gemm_qa_noalloc refuses what does not fit its static scratch array, and MXINT8, before any HIP call."""
    p = 0x1000
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    f = L.mx_gemm_qa_noalloc
    f.argtypes = [i64, i64, i64, vp, i64, ci, ci, vp, vp, ci, vp, ci, i64, vp]
    assert f(8192, 256, 4096, p, 4096, 0, 0, p, p, 0, None, 0, 256, None) == 1          # fits; C is NULL
    assert f(8192 + 1024, 256, 4096, p, 4096, 0, 0, p, p, 0, p, 0, 256, None) == 7       # 37.1 MiB > 36 MiB
    assert f(16384, 256, 4096, p, 4096, 4, 0, p, p, 0, None, 0, 256, None) == 1          # 4-bit: 34 MiB fits
    assert f(256, 256, 512, p, 512, 5, 0, p, p, 5, p, 0, 256, None) == 5                 # MXINT8
    assert f(256, 256, 500, p, 512, 0, 0, p, p, 0, p, 0, 256, None) == 3
    assert f(256, 256, 512, p, 512, 0, 3, p, p, 0, p, 0, 256, None) == 2                 # stochastic rounding
    assert f(0, 256, 512, None, 512, 0, 0, None, None, 0, None, 0, 256, None) == 0
    assert b"scratch" in L.mx_strerror(7)


def test_quantize_3d_validation(L):
    p = 0x1000
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    f = L.mx_quantize_3d
    f.argtypes = [vp, ci, i64, i64, i64, i64, i64, ci, ci, ci, ci, vp, vp, vp]
    assert f(p, 1, 2, 32, 64, 2048, 64, 3, 0, 0, 0, p, p, None) == 2        # axis
    assert f(p, 1, 2, 32, 64, 2048, 64, 1, 0, 3, 0, p, p, None) == 2        # stochastic rounding
    assert f(p, 1, 2, 32, 64, 2048, 32, 1, 0, 0, 0, p, p, None) == 3        # stride1 < d2
    assert f(p, 1, 2, 32, 64, 1024, 64, 1, 0, 0, 0, p, p, None) == 3        # stride0 < d1 * stride1
    assert f(p, 1, 2, 32, 6, 2048, 64, 1, 2, 0, 1, p, p, None) == 3         # 6 codes of 6 bits do not end on a byte
    assert f(p, 1, 2, 32, 6, 2048, 64, 1, 2, 0, 0, None, p, None) == 1      # fine in the block-major layout
    assert f(p, 1, 2, 32, 64, 4352, 68, 1, 0, 0, 0, p, p, None) == 4        # 68 bf16 = 136 bytes per row
    assert f(None, 1, 0, 32, 64, 2048, 64, 1, 0, 0, 0, None, None, None) == 0


def test_workspace_queries_and_validation(L):
    from paper_2310_10537_amd import binding
    wb = binding.mx_workspace_bytes
    assert wb("gemm", 8192, 4096, 4096, 0, 0) == 0                       # FP8 operands never need scratch
    assert wb("gemm", 8192, 4096, 4096, 5, 5) >= (8192 + 4096) * 128 * 100
    assert wb("gemm_qa", 8192, 4096, 4096, 0, 0) >= 8192 * 4096 * (1 + 1 / 32)
    assert wb("gemm_qa", 8192, 4096, 4096, 4, 0) < wb("gemm_qa", 8192, 4096, 4096, 0, 0)
    assert wb("gemm_q", 300, 520, 640, 0, 3) >= 300 * 520 * 4
    p = 0x1000
    # a workspace below the bound is refused before anything is launched
    assert L.mx_gemm_qa_ws(8192, 4096, 4096, p, 4096, 0, 0, p, p, 0, p, 1, 4096, p, 1024, None) == 8
    assert L.mx_gemm_ws(8192, 4096, 4096, p, p, 5, p, p, 5, p, 1, 4096, p, 4096, None) == 8
    assert L.mx_gemm_q_ws(300, 520, 640, p, p, 0, p, p, 3, 2, 0, p, p, p, 100, None) == 8
    assert L.mx_gemm_qa_ws(8192, 4096, 4096, p, 4096, 0, 0, p, p, 0, p, 1, 4096, p + 8, 1 << 30, None) == 4
    assert b"workspace" in L.mx_strerror(8)


def test_gemm_probe_validation(L):
    p = 0x1000
    args = lambda M, N, K, fa, fb, plen: (M, N, K, p, p, fa, p, p, fb, p, N, p, plen, None)
    assert L.mx_gemm_probe(*args(512, 512, 512, 0, 1, 64)) == 5          # pair without a probe build
    assert L.mx_gemm_probe(*args(500, 512, 512, 0, 0, 64)) == 3          # whole tiles only
    assert L.mx_gemm_probe(*args(512, 512, 256, 0, 0, 64)) == 3
    assert L.mx_gemm_probe(*args(512, 512, 512, 0, 0, 8)) == 3           # probe buffer too short
    assert L.mx_gemm_probe(512, 512, 512, p, p, 0, p, p, 0, p, 512, None, 64, None) == 1


def test_mfma_stream_probe_validation(L):
    p = 0x1000
    f = L.mx_mfma_stream_probe
    assert f(5, p, 10, p, p, None) == 5          # INT8 has no such instruction
    assert f(0, p, 0, p, p, None) == 3
    assert f(0, p, (1 << 20) + 1, p, p, None) == 3
    assert f(0, None, 10, p, p, None) == 1
    assert f(0, p + 16, 10, p, p, None) == 4     # operand registers are loaded 32 bytes at a time


def test_dequantize_3d_validation(L):
    p = 0x1000
    ok = (p, p, 0, 4, 6, 64, 1, 0, p, 0, 6 * 64, 64, None)
    bad = lambda **kw: tuple(kw.get(k, v) for k, v in zip("elems scales fmt d0 d1 d2 axis keep dst dt s0 s1 st".split(), ok))
    assert L.mx_dequantize_3d(*bad(axis=3)) == 2
    assert L.mx_dequantize_3d(*bad(keep=2)) == 2
    assert L.mx_dequantize_3d(*bad(s1=60)) == 3
    assert L.mx_dequantize_3d(*bad(s0=5 * 64)) == 3
    assert L.mx_dequantize_3d(*bad(fmt=2, d2=65, s1=80, s0=480, keep=1)) == 3      # 65 six-bit codes are no whole bytes
    assert L.mx_dequantize_3d(*bad(d0=0)) == 0
    assert L.mx_dequantize_3d(*bad(dst=None)) == 1
    assert L.mx_dequantize_3d(*bad(s1=66, s0=6 * 66)) == 4                          # Float32 rows must start 16-byte aligned
