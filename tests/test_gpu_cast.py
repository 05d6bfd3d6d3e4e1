"""GPU parity of mx_quantize / mx_dequantize against the CPU reference:
bit-exact element bytes and scale bytes on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2310_10537_amd import inputs

pytestmark = pytest.mark.gpu

FORMATS = range(6)
NAMES = ("fp8_e4m3", "fp8_e5m2", "fp6_e3m2", "fp6_e2m3", "fp4_e2m1", "int8")
RNE, AWAY = 0, 1


@pytest.fixture(scope="module")
def mx():
    from paper_2310_10537_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()
    return binding


from gpu_util import same_floats, to_dev, to_host  # noqa: E402


def check_cast(mx, oracle, src_np, axis, fmt, rnd, tag=""):
    e_ref, s_ref = oracle.quantize(src_np, axis, fmt, rnd)
    e, s = mx.mx_quantize(to_dev(src_np), axis, fmt, rnd)
    torch.cuda.synchronize()
    e, s = to_host(e), to_host(s)
    assert e.shape == e_ref.shape and s.shape == s_ref.shape
    bad_s = np.argwhere(s != s_ref)
    assert bad_s.size == 0, f"{tag} scale mismatch at {bad_s[:5].tolist()}: got {s[tuple(bad_s[0])]} want {s_ref[tuple(bad_s[0])]}"
    bad_e = np.argwhere(e != e_ref)
    assert bad_e.size == 0, f"{tag} element byte mismatch at {bad_e[:5].tolist()}: got {e[tuple(bad_e[0])]} want {e_ref[tuple(bad_e[0])]}"
    return e_ref, s_ref


def test_config1_roundtrip_fp32_e4m3(mx, oracle):
    """1024 x 1024 float32 N(0,1), seed 0, MXFP8 E4M3, block 32 along the last dim:
    cast, dequantize, and cast again (idempotence on the GPU)."""
    x = inputs.gaussian_f32((1024, 1024), seed=0)
    e_ref, s_ref = check_cast(mx, oracle, x, 1, 0, RNE, "config1")
    e, s = mx.mx_quantize(to_dev(x), 1, 0, RNE)
    y = mx.mx_dequantize(e, s, 0, 1024, 1024, 1)
    y_ref = oracle.dequantize(e_ref, s_ref, 0, 1024, 1024, 1)
    assert same_floats(to_host(y), y_ref)
    e2, s2 = mx.mx_quantize(y, 1, 0, RNE)
    assert torch.equal(e2, e) and torch.equal(s2, s)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_cast_axis1_ragged(mx, oracle, fmt, rnd, dt):
    # 203 rows x 13 blocks: several work-group tiles plus a ragged tail in both dimensions
    x = inputs.student_t_f32((203, 416), seed=10 + fmt)
    src = x if dt == "f32" else inputs.f32_to_bf16_bits(x)
    check_cast(mx, oracle, src, 1, fmt, rnd)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_cast_axis0_ragged(mx, oracle, fmt, rnd, dt):
    # 160 rows (5 blocks) x 200 columns: not a multiple of the column tile
    x = inputs.student_t_f32((160, 200), seed=20 + fmt)
    src = x if dt == "f32" else inputs.f32_to_bf16_bits(x)
    check_cast(mx, oracle, src, 0, fmt, rnd)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
@pytest.mark.parametrize("axis", [1, 0])
def test_cast_adversarial(mx, oracle, fmt, rnd, axis):
    """All-zero, single-outlier, all-equal, exact ties, Float32 subnormals, +-Inf,
    NaN, largest finite, -0 and full-exponent-range blocks."""
    x = inputs.adversarial_f32(256, 512, seed=3)
    if axis == 0:
        x = np.ascontiguousarray(x.T)   # blocks now run down the columns
    check_cast(mx, oracle, x, axis, fmt, rnd)
    xb = inputs.f32_to_bf16_bits(x)
    check_cast(mx, oracle, xb, axis, fmt, rnd)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
def test_cast_exhaustive_bf16(mx, oracle, fmt, rnd):
    """Every bf16 bit pattern, each placed in blocks whose maximum is set by a
    second value sweeping the exponent range, so that every pattern is seen at
    many positions of the element grid (normal, subnormal, underflow, clamp)."""
    pats = np.arange(65536, dtype=np.uint16)
    tops = np.array([0x0080, 0x0C00, 0x3000, 0x3F80, 0x3FC0, 0x4780, 0x5F80, 0x7F7F], dtype=np.uint16)
    src = np.zeros((65536, len(tops) * 32), dtype=np.uint16)
    for j, t in enumerate(tops):
        src[:, 32 * j] = pats
        src[:, 32 * j + 1] = t
        src[:, 32 * j + 2] = pats ^ 0x8000
    check_cast(mx, oracle, src, 1, fmt, rnd)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
def test_cast_fp32_midpoints(mx, oracle, fmt):
    """Float32 inputs sitting exactly on, one ulp below and one ulp above every
    rounding boundary of the element grid, at several scales."""
    w_max = {0: 448.0, 1: 57344.0, 2: 28.0, 3: 7.5, 4: 6.0, 5: 127 / 64}[fmt]
    vals = sorted({abs(oracle.decode(fmt, c)) for c in range(1 << [8, 8, 6, 6, 4, 8][fmt])
                   if np.isfinite(oracle.decode(fmt, c))})
    mids = np.array([(a + b) / 2 for a, b in zip(vals, vals[1:])] + vals[1:], dtype=np.float32)
    pts = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(np.inf))])
    pts = np.concatenate([pts, -pts]).astype(np.float32)
    n = (pts.size + 29) // 30
    blocks = np.zeros((n, 32), dtype=np.float32)
    blocks[:, 0] = np.float32(2.0 ** np.floor(np.log2(w_max)))   # pins X = 1
    flat = np.zeros(n * 30, dtype=np.float32)
    flat[: pts.size] = pts
    blocks[:, 2:] = flat.reshape(n, 30)
    rows = []
    for sc in (0.0, -20.0, 37.0, -100.0):
        rows.append(blocks * np.float32(2.0 ** sc))
    x = np.concatenate(rows, axis=0)
    pad = (-x.shape[0]) % 8
    x = np.concatenate([x, np.zeros((pad, 32), dtype=np.float32)])
    x = np.ascontiguousarray(x.reshape(-1, 256))
    for rnd in (RNE, AWAY):
        check_cast(mx, oracle, x, 1, fmt, rnd)
    # the same blocks running down the columns of a tensor made of whole 128 x 64 tiles: the
    # Float32 column kernel, whose block quantizer is the one the GEMM epilogue uses as well
    x = np.concatenate([x, np.zeros(((-x.shape[0]) % 64, 256), dtype=np.float32)])
    xt = np.ascontiguousarray(x.T)
    assert xt.shape[0] % 128 == 0 and xt.shape[1] % 64 == 0
    for rnd in (RNE, AWAY):
        check_cast(mx, oracle, xt, 0, fmt, rnd, "axis 0 tiles")


def test_cast_random_bits_fp32(mx, oracle):
    # 2^22 random Float32 bit patterns per format (any exponent, NaN/Inf/subnormals included)
    rng = np.random.default_rng(77)
    x = rng.integers(0, 2**32, size=(2048, 2048), dtype=np.uint64).astype(np.uint32).view(np.float32)
    for fmt in FORMATS:
        check_cast(mx, oracle, x, 1, fmt, RNE if fmt % 2 == 0 else AWAY)


def test_cast_leading_dimension(mx, oracle):
    x = inputs.student_t_f32((64, 256), seed=31)
    wide = torch.zeros((64, 320), dtype=torch.float32, device="cuda")
    wide[:, :256] = to_dev(x)
    for axis in (1, 0):
        e, s = mx.mx_quantize(wide[:, :256], axis, 2, AWAY)
        e_ref, s_ref = oracle.quantize(x, axis, 2, AWAY)
        assert np.array_equal(to_host(e), e_ref) and np.array_equal(to_host(s), s_ref)


def test_cast_empty_and_single_block(mx, oracle):
    e, s = mx.mx_quantize(torch.zeros((0, 64), device="cuda"), 1, 0)
    assert e.shape == (0, 64) and s.shape == (0, 2)
    e, s = mx.mx_quantize(torch.zeros((32, 0), device="cuda"), 0, 4)
    assert e.numel() == 0 and s.numel() == 0
    x = inputs.gaussian_f32((1, 32), seed=1)
    col = torch.zeros((32, 4), dtype=torch.float32, device="cuda")   # one column inside a 16-byte-aligned row pitch
    col[:, 0] = to_dev(x)[0]
    for fmt in FORMATS:
        e_ref, s_ref = check_cast(mx, oracle, x, 1, fmt, RNE)
        e, s = mx.mx_quantize(col[:, :1], 0, fmt, RNE)
        assert np.array_equal(to_host(e), e_ref) and np.array_equal(to_host(s), s_ref)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("axis", [1, 0])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n_out", [72, 192], ids=["lines72", "lines192"])
def test_dequantize(mx, oracle, fmt, axis, dt, n_out):
    """Every element code at a sweep of scale bytes (including 0, 254 and the NaN
    scale 0xFF), both orientations; 192 lines x 256 positions are whole 64 x 128 tiles
    of the LDS-transposing axis-0 kernel, 72 lines take the generic one."""
    w = [8, 8, 6, 6, 4, 8][fmt]
    rng = np.random.default_rng(fmt)
    length = 256
    codes = rng.integers(0, 1 << w, size=(n_out, length), dtype=np.uint32)
    codes[0, : 1 << w] = np.arange(1 << w)[:length]
    bits = ((codes[..., None] >> np.arange(w, dtype=np.uint32)) & 1).astype(np.uint8)
    elems = np.packbits(bits.reshape(n_out, -1), axis=-1, bitorder="little")
    scales = rng.integers(0, 256, size=(n_out, length // 32), dtype=np.uint64).astype(np.uint8)
    scales[1, :] = [0, 1, 2, 126, 127, 253, 254, 255]
    rows, cols = (n_out, length) if axis == 1 else (length, n_out)
    ref = oracle.dequantize(elems, scales, fmt, rows, cols, axis, dst_dt=0 if dt == torch.float32 else 1)
    got = mx.mx_dequantize(to_dev(elems), to_dev(scales), fmt, rows, cols, axis, dtype=dt)
    assert same_floats(to_host(got), ref)
    # into a view with a leading dimension: the columns beyond stay untouched
    wide = torch.full((rows, cols + 8), 7.0, dtype=dt, device="cuda")
    mx.mx_dequantize(to_dev(elems), to_dev(scales), fmt, rows, cols, axis, out=wide[:, :cols])
    assert same_floats(to_host(wide[:, :cols].contiguous()), ref) and torch.all(wide[:, cols:] == 7.0)


def test_full_size_config2_sampled(mx, oracle):
    """8192 x 8192 bf16 heavy-tailed activations (the benchmark workload), all six
    formats and both axes, in the launch configuration the benchmark times.
    The reference is evaluated on a sample of 192 rows (axis 1) / columns (axis 0)."""
    x = inputs.student_t_bf16((8192, 8192), seed=1)
    xd = to_dev(x)
    rng = np.random.default_rng(5)
    pick = np.sort(rng.choice(8192, 192, replace=False))
    pick[0], pick[-1] = 0, 8191
    for fmt in FORMATS:
        for axis in (1, 0):
            rnd = AWAY if (fmt == 2 and axis == 0) else RNE
            e, s = mx.mx_quantize(xd, axis, fmt, rnd)
            torch.cuda.synchronize()
            sub = np.ascontiguousarray(x[pick, :] if axis == 1 else x[:, pick])
            e_ref, s_ref = oracle.quantize(sub, axis, fmt, rnd)
            pk = torch.from_numpy(pick).cuda()
            assert np.array_equal(to_host(e[pk]), e_ref), (fmt, axis)
            assert np.array_equal(to_host(s[pk]), s_ref), (fmt, axis)
            # whole-tensor property: no NaN scale and every scale within the data's exponent range
            assert int(s.max()) < 255

@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("shape", [(384, 192), (4128, 4104), (4096, 4096)], ids=["whole_64", "ragged_128", "whole_128"])
def test_cast_axis0_bf16_tile_variants(mx, oracle, fmt, shape):
    """The axis-0 kernel for bf16 sources has four forms: 64- or 128-column tiles, with or without bounds
    checks (every tile inside the tensor).  One shape per form not covered elsewhere; the reference is
    evaluated on a sample of columns that includes the first and the last."""
    x = inputs.student_t_bf16(shape, seed=40 + fmt)
    rnd = AWAY if fmt in (1, 3) else RNE
    e, s = mx.mx_quantize(to_dev(x), 0, fmt, rnd)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    pick = np.sort(rng.choice(shape[1], min(shape[1], 160), replace=False))
    pick[0], pick[-1] = 0, shape[1] - 1
    e_ref, s_ref = oracle.quantize(np.ascontiguousarray(x[:, pick]), 0, fmt, rnd)
    pk = torch.from_numpy(pick).cuda()
    assert np.array_equal(to_host(s[pk]), s_ref), (fmt, shape)
    assert np.array_equal(to_host(e[pk]), e_ref), (fmt, shape)


@pytest.mark.parametrize("fmt", range(6), ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
@pytest.mark.parametrize("shape,kind", [((512, 256), "student"), ((256, 448), "adversarial"), ((128, 64), "student"),
                                        ((96, 160), "student")])
def test_quantize_dual_matches_reference_on_both_axes(mx, oracle, fmt, rnd, shape, kind):
    """One pass, two MX tensors: each must be byte-identical to the reference cast along its axis.
    Whole 128 x 64 tiles take the one-pass kernel (degenerate blocks included), the last shape the
    two-launch fallback."""
    rows, cols = shape
    if kind == "adversarial":
        x = inputs.f32_to_bf16_bits(inputs.adversarial_f32(rows, cols, seed=31 + fmt))
    else:
        x = inputs.student_t_bf16((rows, cols), seed=30 + fmt)
    (e1, s1), (e0, s0) = mx.mx_quantize_dual(to_dev(x), fmt, rnd)
    for axis, e, s in ((1, e1, s1), (0, e0, s0)):
        re_, rs = oracle.quantize(x, axis, fmt, rnd)
        assert np.array_equal(to_host(s), rs), f"scales axis {axis}"
        assert np.array_equal(to_host(e), re_), f"elements axis {axis}"


def test_quantize_dual_fp32_source_and_leading_dimension(mx, oracle):
    """fp32 sources and padded rows go through the two ordinary casts; a bf16 view with a leading
    dimension still takes the one-pass kernel."""
    x = inputs.gaussian_f32((128, 192), seed=33)
    (e1, s1), (e0, s0) = mx.mx_quantize_dual(to_dev(x), 2)
    for axis, e, s in ((1, e1, s1), (0, e0, s0)):
        re_, rs = oracle.quantize(x, axis, 2, 0)
        assert np.array_equal(to_host(s), rs) and np.array_equal(to_host(e), re_)
    big = inputs.student_t_bf16((256, 256), seed=34)
    view = to_dev(big)[:, 64:192]
    (e1, s1), (e0, s0) = mx.mx_quantize_dual(view, 0)
    sub = np.ascontiguousarray(big[:, 64:192])
    for axis, e, s in ((1, e1, s1), (0, e0, s0)):
        re_, rs = oracle.quantize(sub, axis, 0, 0)
        assert np.array_equal(to_host(s), rs) and np.array_equal(to_host(e), re_)


def test_quantize_dual_full_size_sampled(mx, oracle):
    """The 8192 x 8192 workload tensor: slices of both outputs against the reference."""
    x = inputs.student_t_bf16((8192, 8192), seed=1)
    (e1, s1), (e0, s0) = mx.mx_quantize_dual(to_dev(x), 0)
    for lo in (0, 4000, 8192 - 128):
        re_, rs = oracle.quantize(np.ascontiguousarray(x[lo:lo + 128]), 1, 0, 0)
        assert np.array_equal(to_host(e1[lo:lo + 128]), re_) and np.array_equal(to_host(s1[lo:lo + 128]), rs)
        re_, rs = oracle.quantize(np.ascontiguousarray(x[:, lo:lo + 128]), 0, 0, 0)
        assert np.array_equal(to_host(e0[lo:lo + 128]), re_) and np.array_equal(to_host(s0[lo:lo + 128]), rs)

@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
def test_quantize_dual_wide_tiles_all_formats(mx, oracle, fmt):
    """4096 x 4096: the dual-axis kernel's 128-column tiles (FP6: its 16-byte store paths) in every format,
    slices of both outputs against the reference."""
    x = inputs.student_t_bf16((4096, 4096), seed=50 + fmt)
    rnd = AWAY if fmt in (2, 5) else RNE
    (e1, s1), (e0, s0) = mx.mx_quantize_dual(to_dev(x), fmt, rnd)
    for lo in (0, 1984, 4096 - 160):
        re_, rs = oracle.quantize(np.ascontiguousarray(x[lo:lo + 160]), 1, fmt, rnd)
        assert np.array_equal(to_host(s1[lo:lo + 160]), rs) and np.array_equal(to_host(e1[lo:lo + 160]), re_), (fmt, lo, "axis 1")
        re_, rs = oracle.quantize(np.ascontiguousarray(x[:, lo:lo + 160]), 0, fmt, rnd)
        assert np.array_equal(to_host(s0[lo:lo + 160]), rs) and np.array_equal(to_host(e0[lo:lo + 160]), re_), (fmt, lo, "axis 0")


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_dequantize_every_code_at_every_scale(mx, oracle, fmt, dt):
    """Row r carries scale byte r (0 .. 255, the last one the NaN scale) in all its blocks, and
    every element code of the format appears in every row: all (code, scale) pairs, including the
    products that overflow Float32 or fall into the subnormal range of the output type."""
    w = [8, 8, 6, 6, 4, 8][fmt]
    length = 256
    codes = np.tile(np.arange(length, dtype=np.uint32) % (1 << w), (256, 1))
    bits = ((codes[..., None] >> np.arange(w, dtype=np.uint32)) & 1).astype(np.uint8)
    elems = np.packbits(bits.reshape(256, -1), axis=-1, bitorder="little")
    scales = np.repeat(np.arange(256, dtype=np.uint8)[:, None], length // 32, axis=1)
    ref = oracle.dequantize(elems, scales, fmt, 256, length, 1, dst_dt=0 if dt == torch.float32 else 1)
    got = to_host(mx.mx_dequantize(to_dev(elems), to_dev(scales), fmt, 256, length, 1, dtype=dt))
    if dt == torch.float32:
        same = (got.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(got) & np.isnan(ref))
    else:
        same = (got == ref) | (((got & 0x7FFF) > 0x7F80) & ((ref & 0x7FFF) > 0x7F80))
    rows_bad = np.unique(np.nonzero(~same)[0])
    assert same.all(), f"mismatches at scale bytes {rows_bad[:20]} (first code {np.nonzero(~same)[1][:5]})"


# ---------------------------------------------------------------------------------------------
# The two added rounding modes: magnitude truncation and stochastic rounding.
# ---------------------------------------------------------------------------------------------
RTZ, SR = 2, 3


def dev_view(src_np):
    """Device tensor of src_np as a view into a wider allocation when its row length is not a
    16-byte multiple (the library wants aligned rows, not aligned column counts)."""
    rows, cols = src_np.shape
    pad = (-cols) % 8
    if pad == 0:
        return to_dev(src_np)
    wide = np.zeros((rows, cols + pad), dtype=src_np.dtype)
    wide[:, :cols] = src_np
    return to_dev(wide)[:, :cols]


def check_cast_sr(mx, oracle, src_np, axis, fmt, seed, tag=""):
    e_ref, s_ref = oracle.quantize(src_np, axis, fmt, SR, seed=seed)
    e, s = mx.mx_quantize_sr(dev_view(src_np), axis, fmt, seed)
    torch.cuda.synchronize()
    e, s = to_host(e), to_host(s)
    assert np.array_equal(s, s_ref), f"{tag} scale bytes differ"
    bad = np.argwhere(e != e_ref)
    assert bad.size == 0, f"{tag} element byte mismatch at {bad[:5].tolist()}: got {e[tuple(bad[0])]} want {e_ref[tuple(bad[0])]}"
    return e_ref, s_ref


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("axis,shape", [(1, (203, 416)), (0, (160, 200)), (0, (96, 203))], ids=["axis1", "axis0", "axis0_odd_cols"])
def test_cast_toward_zero(mx, oracle, fmt, dt, axis, shape):
    x = inputs.student_t_f32(shape, seed=60 + fmt)
    src = x if dt == "f32" else inputs.f32_to_bf16_bits(x)
    e_ref, s_ref = oracle.quantize(src, axis, fmt, RTZ)
    e, s = mx.mx_quantize(dev_view(src), axis, fmt, RTZ)
    assert np.array_equal(to_host(s), s_ref) and np.array_equal(to_host(e), e_ref)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("axis,shape", [(1, (203, 416)), (0, (160, 200)), (0, (96, 204)), (0, (64, 203))],
                         ids=["axis1", "axis0", "axis0_cols_204", "axis0_odd_cols"])
def test_cast_stochastic(mx, oracle, fmt, dt, axis, shape):
    """Bit-exact against the reference: same generator, same element numbering, same arithmetic.
    Column counts that are and are not multiples of 4 take the two ways the axis-0 kernel draws
    its numbers."""
    x = inputs.student_t_f32(shape, seed=70 + fmt)
    src = x if dt == "f32" else inputs.f32_to_bf16_bits(x)
    check_cast_sr(mx, oracle, src, axis, fmt, seed=0x9E3779B97F4A7C15 + fmt)
    check_cast_sr(mx, oracle, src, axis, fmt, seed=1)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("mode", ["rtz", "sr"])
@pytest.mark.parametrize("axis", [1, 0])
def test_added_modes_adversarial(mx, oracle, fmt, mode, axis):
    """All-zero, single-outlier, exact ties, Float32 subnormals, +-Inf, NaN, largest finite, -0 and
    full-exponent-range blocks under the two added modes."""
    x = inputs.adversarial_f32(256, 512, seed=4)
    if axis == 0:
        x = np.ascontiguousarray(x.T)
    if mode == "rtz":
        check_cast(mx, oracle, x, axis, fmt, RTZ)
    else:
        check_cast_sr(mx, oracle, x, axis, fmt, seed=77)


def test_stochastic_leading_dimension_and_large_index(mx, oracle):
    """A source view with ld > cols numbers its elements by (row, col), not by address; a tall
    tensor takes the element counter past 2^25."""
    full = inputs.gaussian_f32((128, 160), seed=80)
    view = to_dev(full)[:, :96]
    e, s = mx.mx_quantize_sr(view, 1, 0, 5)
    e_ref, s_ref = oracle.quantize(np.ascontiguousarray(full[:, :96]), 1, 0, SR, seed=5)
    assert np.array_equal(to_host(e), e_ref) and np.array_equal(to_host(s), s_ref)
    e, s = mx.mx_quantize_sr(view, 0, 0, 5)
    e_ref, s_ref = oracle.quantize(np.ascontiguousarray(full[:, :96]), 0, 0, SR, seed=5)
    assert np.array_equal(to_host(e), e_ref) and np.array_equal(to_host(s), s_ref)
    tall = inputs.gaussian_bf16((8192, 4160), seed=81)          # 34 M elements
    for axis in (1, 0):
        e, s = mx.mx_quantize_sr(to_dev(tall), axis, 4, 9)
        e_ref, s_ref = oracle.quantize(tall, axis, 4, SR, seed=9)
        assert np.array_equal(to_host(e), e_ref) and np.array_equal(to_host(s), s_ref)


def test_stochastic_is_unbiased_on_the_gpu(mx, oracle):
    """Mean of dequantized casts over seeds approaches the input; round-to-nearest does not move."""
    x = inputs.gaussian_f32((64, 256), seed=82)
    xd = to_dev(x)
    acc = torch.zeros_like(xd, dtype=torch.float64)
    n = 64
    for seed in range(n):
        e, s = mx.mx_quantize_sr(xd, 1, 4, seed)            # FP4: the coarsest grid
        acc += mx.mx_dequantize(e, s, 4, 64, 256, 1).double()
    mean = to_host(acc / n)
    e, s = mx.mx_quantize(xd, 1, 4, RNE)
    X = np.exp2(to_host(s).astype(np.float64) - 127).repeat(32, axis=1)
    target = np.clip(x.astype(np.float64), -6 * X, 6 * X)
    assert np.all(np.abs(mean - target) <= 5 * 2 * X / (2 * np.sqrt(n)))
    near = to_host(mx.mx_dequantize(e, s, 4, 64, 256, 1)).astype(np.float64)
    assert np.abs(mean - target).mean() < 0.5 * np.abs(near - target).mean()


def test_gemm_qa_toward_zero(mx, oracle):
    """mx_gemm_qa with truncation = truncating cast + mx_gemm, on a tiled and on a ragged shape."""
    for (M, N, K) in ((256, 256, 512), (100, 72, 96)):
        a = inputs.student_t_bf16((M, K), seed=83)
        b = inputs.gaussian_f32((N, K), seed=84, std=0.02)
        for fa in (0, 3, 5):
            fb = 5 if fa == 5 else 0
            gb = mx.mx_quantize(to_dev(b), 1, fb)
            ga = mx.mx_quantize(to_dev(a), 1, fa, RTZ)
            ea, sa = oracle.quantize(a, 1, fa, RTZ)
            assert np.array_equal(to_host(ga[0]), ea) and np.array_equal(to_host(ga[1]), sa)
            C2 = mx.mx_gemm(ga[0], ga[1], fa, gb[0], gb[1], fb, K)
            C1 = mx.mx_gemm_qa(to_dev(a), fa, RTZ, gb[0], gb[1], fb)
            assert torch.equal(C1.view(torch.int32), C2.view(torch.int32))
    with pytest.raises(mx.MxError):
        mx.mx_gemm_qa(to_dev(a), 0, SR, gb[0], gb[1], 0)


# ---------------------------------------------------------------------------------------------
# Block-axis lengths that are not multiples of 32: the last block is filled with zeros.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("axis,shape", [(1, (67, 100)), (1, (5, 31)), (1, (40, 1)), (1, (33, 203)), (0, (100, 72)), (0, (31, 40)),
                                        (0, (1, 8)), (0, (203, 41))],
                         ids=lambda v: str(v).replace(" ", ""))
def test_partial_last_block(mx, oracle, fmt, dt, axis, shape):
    x = inputs.student_t_f32(shape, seed=90 + fmt)
    src = x if dt == "f32" else inputs.f32_to_bf16_bits(x)
    dev = dev_view(src)
    for rnd in (RNE, AWAY, RTZ):
        e_ref, s_ref = oracle.quantize(src, axis, fmt, rnd)
        e, s = mx.mx_quantize(dev, axis, fmt, rnd)
        assert e.shape == e_ref.shape and s.shape == s_ref.shape
        assert np.array_equal(to_host(s), s_ref) and np.array_equal(to_host(e), e_ref), rnd
    e_ref, s_ref = oracle.quantize(src, axis, fmt, SR, seed=21)
    e, s = mx.mx_quantize_sr(dev, axis, fmt, 21)
    assert np.array_equal(to_host(s), s_ref) and np.array_equal(to_host(e), e_ref)
    # and back: only the positions of the tensor are written
    for out_dt, odt in ((torch.float32, 0), (torch.bfloat16, 1)):
        rows, cols = shape
        pad = (-cols) % 8
        wide = torch.full((rows, cols + pad + 8), 7.0, dtype=out_dt, device="cuda")
        mx.mx_dequantize(e, s, fmt, rows, cols, axis, out=wide[:, :cols])
        ref = oracle.dequantize(e_ref, s_ref, fmt, rows, cols, axis, odt)
        assert same_floats(to_host(wide[:, :cols].contiguous()), ref)
        assert torch.all(wide[:, cols:] == 7.0)


def test_partial_block_tensor_feeds_the_gemm(mx, oracle):
    """An operand with K = 100 is cast into 4 blocks (128 positions); the fill adds nothing."""
    M, N, K = 48, 40, 100
    a = inputs.student_t_bf16((M, K), seed=95)
    b = inputs.gaussian_f32((N, K), seed=96)
    ga = mx.mx_quantize(dev_view(a), 1, 0)
    gb = mx.mx_quantize(dev_view(b), 1, 2)
    C = to_host(mx.mx_gemm(ga[0], ga[1], 0, gb[0], gb[1], 2, 128))
    ea, sa = oracle.quantize(a, 1, 0)
    eb, sb = oracle.quantize(b, 1, 2)
    assert np.array_equal(to_host(ga[0]), ea) and np.array_equal(to_host(gb[0]), eb)
    # the reference product over the 100 real positions = the product over the 128 stored ones
    Ad = oracle.dequantize(ea, sa, 0, M, K, 1).astype(np.float64)
    Bd = oracle.dequantize(eb, sb, 2, N, K, 1).astype(np.float64)
    ref128, abs128 = oracle.gemm(ea, sa, 0, eb, sb, 2, 128, want_abs=True)
    assert np.allclose(ref128, Ad @ Bd.T, rtol=1e-12, atol=0)
    from test_gpu_gemm import check_gemm, hw_term_for
    check_gemm(C, ref128, abs128, "partial block operand", hw_term_for(oracle, ea, sa, 0, eb, sb, 2, 128))


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
def test_cast_axis0_f32_whole_tiles(mx, oracle, fmt, rnd):
    """Float32 sources made of whole 128 x 64 tiles take the LDS-tiled column kernel (weights are cast
    from Float32 along dimension 0): heavy-tailed data with per-block magnitudes over 2^+-30, exact
    ties of every element grid, and a view with a leading dimension."""
    rows, cols = 384, 320
    rng = np.random.default_rng(fmt)
    x = inputs.student_t_f32((rows, cols), seed=97 + fmt)
    x *= np.exp2(rng.integers(-30, 30, (rows // 32, cols))).repeat(32, axis=0).astype(np.float32)
    # ties: k + 0.5 steps of the finest grid around 1.0 of each format, scaled per column block
    x[:32, :64] = ((np.arange(32)[:, None] + 0.5) * 2.0 ** -6 * (1 + np.arange(64)[None, :] % 3)).astype(np.float32)
    x[5, 70] = 0.0
    check_cast(mx, oracle, x, 0, fmt, rnd)
    wide = np.zeros((rows, cols + 64), dtype=np.float32)
    wide[:, :cols] = x
    e, s = mx.mx_quantize(to_dev(wide)[:, :cols], 0, fmt, rnd)
    e_ref, s_ref = oracle.quantize(x, 0, fmt, rnd)
    assert np.array_equal(to_host(e), e_ref) and np.array_equal(to_host(s), s_ref)


@pytest.mark.parametrize("fmt", FORMATS, ids=NAMES)
@pytest.mark.parametrize("rnd", [RNE, AWAY], ids=["rne", "away"])
def test_cast_axis1_f32_dense_runs(mx, oracle, fmt, rnd):
    """Dense Float32 tensors made of whole 2048-element runs take the wave-level row kernel on the hardware
    converts: heavy-tailed data with per-block magnitudes over 2^+-30, exact ties and the values one ulp
    either side of them for every element grid, degenerate blocks (zeros, Inf, NaN, subnormals, largest
    finite), and a shape whose rows are shorter than a run."""
    rows, cols = 96, 1024
    rng = np.random.default_rng(10 + fmt)
    x = inputs.student_t_f32((rows, cols), seed=117 + fmt)
    x *= np.exp2(rng.integers(-30, 30, (rows, cols // 32))).repeat(32, axis=1).astype(np.float32)
    ties = ((np.arange(64) + 0.5) * 2.0 ** -6).astype(np.float32)
    x[0, :64] = ties
    x[1, :64] = np.nextafter(ties, np.float32(0))
    x[2, :64] = np.nextafter(ties, np.float32(4))
    x[3, :64] = -ties
    check_cast(mx, oracle, x, 1, fmt, rnd)
    check_cast(mx, oracle, inputs.adversarial_f32(64, 2048, seed=5 + fmt), 1, fmt, rnd)
    check_cast(mx, oracle, inputs.student_t_f32((1024, 64), seed=3), 1, fmt, rnd)      # 32 rows per run
