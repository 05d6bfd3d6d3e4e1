"""mx_quantize_3d against the reference: Algorithm 1 along any axis of a strided 3-D tensor
(Section 3, principal axis), block-major and source-order output, bit for bit."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev, to_host
from paper_2310_10537_amd import inputs

pytestmark = pytest.mark.gpu
NAMES = ("fp8_e4m3", "fp8_e5m2", "fp6_e3m2", "fp6_e2m3", "fp4_e2m1", "int8")


@pytest.fixture(scope="module")
def mx():
    from paper_2310_10537_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()
    return binding


def check(mx, oracle, x, axis, fmt, rnd, keep, view=None):
    """x: host array (float32 or bf16 bits) [d0, d1, d2]; view: slicing applied on both sides."""
    d = to_dev(x)
    if view is not None:
        d, x = d[view], np.ascontiguousarray(x[view])
    e, s = mx.mx_quantize_3d(d, axis, fmt, rnd, keep)
    torch.cuda.synchronize()
    e_ref, s_ref = oracle.quantize_3d(x, axis, fmt, rnd, keep)
    e, s = to_host(e), to_host(s)
    assert e.shape == e_ref.shape and s.shape == s_ref.shape
    bad = np.argwhere(s != s_ref)
    assert bad.size == 0, f"scale bytes differ at {bad[:4].tolist()}"
    bad = np.argwhere(e != e_ref)
    assert bad.size == 0, f"element bytes differ at {bad[:4].tolist()}: {e[tuple(bad[0])]} vs {e_ref[tuple(bad[0])]}"


@pytest.mark.parametrize("fmt", range(6), ids=NAMES)
@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("keep", [False, True], ids=["block_major", "source_order"])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_every_axis_and_layout(mx, oracle, fmt, axis, keep, dt):
    # two of the three axes end in a partial block; d2 keeps rows byte-aligned for every width
    shape = (40, 70, 24) if keep else (40, 70, 72)
    x = inputs.student_t_f32((shape[0] * shape[1], shape[2]), seed=50 + fmt).reshape(shape)
    src = x if dt == "f32" else inputs.f32_to_bf16_bits(x)
    for rnd in (0, 1, 2):
        check(mx, oracle, src, axis, fmt, rnd, keep)


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("keep", [False, True], ids=["block_major", "source_order"])
def test_whole_tiles_take_the_fast_kernels_per_slice(mx, oracle, axis, keep):
    """A batch of 128 x 256 bf16 matrices (whole tiles for the fast 2-D kernels) and degenerate values."""
    x = inputs.adversarial_f32(4 * 128, 256, seed=9).reshape(4, 128, 256)
    for fmt in (0, 2, 4):
        check(mx, oracle, inputs.f32_to_bf16_bits(x), axis, fmt, 0, keep)
        check(mx, oracle, x, axis, fmt, 1, keep)


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("keep", [False, True], ids=["block_major", "source_order"])
def test_strided_views(mx, oracle, axis, keep):
    """Slices of a larger tensor: both leading strides differ from the dense ones, and the slices'
    scale arrays start at odd addresses inside the output."""
    big = inputs.gaussian_f32((6 * 50, 96), seed=13).reshape(6, 50, 96)
    for fmt in (1, 3, 5):
        check(mx, oracle, big, axis, fmt, 0, keep, view=np.s_[1:5, 8:47, 32:96])
        check(mx, oracle, inputs.f32_to_bf16_bits(big), axis, fmt, 1, keep, view=np.s_[0:3, 0:50, 0:40])


def test_matrix_with_untransposed_axis0_output(mx, oracle):
    """d0 = 1: a plain matrix cast along its rows' direction with the codes left in place."""
    x = inputs.student_t_bf16((2048, 1024), seed=77)
    for fmt in (0, 4):
        check(mx, oracle, x.reshape(1, 2048, 1024), 1, fmt, 0, True)
    e, s = mx.mx_quantize_3d(to_dev(x).reshape(1, 2048, 1024), 1, 0, 0, True)
    et, st = mx.mx_quantize(to_dev(x), 0, 0)              # the transposed form of the same cast
    assert torch.equal(e[0].T.contiguous(), et) and torch.equal(s[0].T.contiguous(), st)


# ---------------------------------------------------------------------------------------------
# mx_dequantize_3d: the inverse, against the reference's mxo_dequantize_3d, bit for bit
# ---------------------------------------------------------------------------------------------
def same_bits(got, want):
    """Float32 arrays (or uint16 bf16 bits): equal bit patterns, NaN matched by position."""
    if got.dtype == np.uint16:
        gn, wn = (got & 0x7FFF) > 0x7F80, (want & 0x7FFF) > 0x7F80
        return np.array_equal(gn, wn) and np.array_equal(got[~gn], want[~wn])
    gn, wn = np.isnan(got), np.isnan(want)
    return np.array_equal(gn, wn) and np.array_equal(got[~gn].view(np.uint32), want[~wn].view(np.uint32))


def check_deq(mx, oracle, x, axis, fmt, keep, dt, out=None, nan_block=False):
    shape = x.shape
    e, s = oracle.quantize_3d(x, axis, fmt, 0, keep)
    if nan_block:
        s = s.copy()
        s.reshape(-1)[s.size // 3] = 255
    want = oracle.dequantize_3d(e, s, fmt, shape, axis, keep, dst_dt=0 if dt == torch.float32 else 1)
    got = mx.mx_dequantize_3d(to_dev(e), to_dev(s), fmt, shape, axis, keep, dtype=dt, out=out)
    torch.cuda.synchronize()
    g = to_host(got.contiguous() if dt == torch.float32 else got.contiguous().view(torch.int16)).view(np.float32 if dt == torch.float32 else np.uint16)
    assert same_bits(g, want), (fmt, axis, keep, dt)


@pytest.mark.parametrize("fmt", range(6), ids=NAMES)
@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("keep", [False, True], ids=["block_major", "source_order"])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_dequantize_every_axis_and_layout(mx, oracle, fmt, axis, keep, dt):
    shape = (40, 70, 24) if keep else (40, 70, 72)      # two axes end in a partial block
    x = inputs.student_t_f32((shape[0] * shape[1], shape[2]), seed=60 + fmt).reshape(shape)
    check_deq(mx, oracle, x, axis, fmt, keep, dt, nan_block=True)


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("keep", [False, True], ids=["block_major", "source_order"])
def test_dequantize_whole_tiles_and_degenerate_values(mx, oracle, axis, keep):
    """4 x 128 x 256: the slices are whole tiles of the fast 2-D dequantize kernels; adversarial blocks."""
    x = inputs.adversarial_f32(4 * 128, 256, seed=19).reshape(4, 128, 256)
    for fmt in (0, 3, 4, 5):
        check_deq(mx, oracle, x, axis, fmt, keep, torch.float32)
        check_deq(mx, oracle, x, axis, fmt, keep, torch.bfloat16)


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("keep", [False, True], ids=["block_major", "source_order"])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_dequantize_into_a_strided_view(mx, oracle, axis, keep, dt):
    """The result is a slice of a larger tensor: both leading strides are padded, and nothing outside the
    slice may be written."""
    shape = (3, 37, 64)
    x = inputs.gaussian_f32((3 * 37, 64), seed=23).reshape(shape)
    big = torch.full((5, 48, 96), 7.0, dtype=dt, device="cuda")
    view = big[1:4, 8:45, 32:96]
    for fmt in (1, 2, 4):
        check_deq(mx, oracle, x, axis, fmt, keep, dt, out=view)
        mask = torch.ones_like(big, dtype=torch.bool)
        mask[1:4, 8:45, 32:96] = False
        assert torch.all(big[mask] == 7.0)


def test_round_trip_with_the_gpu_cast(mx, oracle):
    """quantize_3d then dequantize_3d on the GPU, both layouts: the same tensor, and casting it again
    returns the same bytes (idempotence)."""
    x = to_dev(inputs.student_t_bf16((6 * 96, 128), seed=31)).reshape(6, 96, 128)
    for axis in (0, 1, 2):
        outs = []
        for keep in (False, True):
            e, s = mx.mx_quantize_3d(x, axis, 0, 0, keep)
            y = mx.mx_dequantize_3d(e, s, 0, (6, 96, 128), axis, keep, dtype=torch.bfloat16)
            e2, s2 = mx.mx_quantize_3d(y, axis, 0, 0, keep)
            assert torch.equal(e, e2) and torch.equal(s, s2)
            outs.append(y)
        assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
