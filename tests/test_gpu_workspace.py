"""The GEMM entry points that take their scratch memory from a caller-owned workspace (mx_gemm_ws,
mx_gemm_qa_ws, mx_gemm_q_ws) against the ones that take it from the memory pool: the same bytes, on every
route that needs scratch, with a workspace of exactly the size the library asks for, poisoned beforehand;
and a workspace that is one byte short is refused with nothing launched."""
import pytest
import torch

from gpu_util import to_dev
from paper_2310_10537_amd import inputs

pytestmark = pytest.mark.gpu

FP8, E5M2, E3M2, E2M3, FP4, INT8 = 0, 1, 2, 3, 4, 5


@pytest.fixture(scope="module")
def mx():
    from paper_2310_10537_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()
    return binding


def bits_equal(a, b):
    v = {torch.bfloat16: torch.int16, torch.float32: torch.int32, torch.uint8: torch.uint8}[a.dtype]
    return torch.equal(a.view(v), b.view(v))


def workspace(n):
    # poisoned: a route that read scratch it had not written would not reproduce the pool-based result
    return torch.full((max(n, 16),), 0xA5, dtype=torch.uint8, device="cuda")


def operands(mx, M, N, K, fa, fb, seed):
    a = to_dev(inputs.student_t_bf16((M, K), seed=seed))
    b = to_dev(inputs.gaussian_f32((N, K), seed=seed + 1, std=0.02))
    return a, mx.mx_quantize(a, 1, fa), mx.mx_quantize(b, 1, fb)


QA_CASES = [
    # the transformer projection: cast into scratch, then the LDS-tiled kernel
    ("proj_fp8", 8192, 4096, 4096, FP8, FP8, 0, torch.bfloat16),
    ("tiled_fp4_away", 2048, 1024, 1024, FP4, E3M2, 1, torch.float32),
    ("tiled_trunc", 1024, 512, 512, FP8, FP8, 2, torch.float32),        # toward zero always casts first
    ("few_rows", 64, 1024, 1024, E2M3, FP8, 0, torch.float32),          # shared-K kernel
    ("ragged", 300, 520, 640, FP8, FP4, 0, torch.float32),              # interior + fringes, cast once
    ("int8", 512, 256, 512, INT8, INT8, 0, torch.float32),              # per-block integer kernel
    ("int8_split", 4096, 4096, 1024, INT8, INT8, 0, torch.bfloat16),    # cast + the two E2M3 halves
]


@pytest.mark.parametrize("case", QA_CASES, ids=[c[0] for c in QA_CASES])
def test_gemm_qa_ws_matches_pool_route(mx, case):
    _, M, N, K, fa, fb, rnd, dt = case
    a, _, gb = operands(mx, M, N, K, fa, fb, 300)
    need = mx.mx_workspace_bytes("gemm_qa", M, N, K, fa, fb)
    assert need > 0
    want = mx.mx_gemm_qa(a, fa, rnd, gb[0], gb[1], fb, dtype=dt)
    ws = workspace(need)
    out = torch.full((M, N), 7.0, dtype=dt, device="cuda")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    mx.mx_gemm_qa_ws(a, fa, rnd, gb[0], gb[1], fb, ws[:need], out=out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before                   # nothing was taken from the device
    assert bits_equal(out, want)
    # one byte short: refused before anything runs
    out.fill_(7.0)
    with pytest.raises(mx.MxError) as err:
        mx.mx_gemm_qa_ws(a, fa, rnd, gb[0], gb[1], fb, ws[:need - 1], out=out)
    assert err.value.status == mx.MX_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)
    # no workspace: the pool route
    assert bits_equal(mx.mx_gemm_qa_ws(a, fa, rnd, gb[0], gb[1], fb, None, dtype=dt), want)


@pytest.mark.parametrize("shape", [(4096, 4096, 1024), (2304, 2816, 512)], ids=["256_tiles", "99_tiles_short_k"])
def test_int8_split_ws_matches_pool_route(mx, shape):
    M, N, K = shape
    _, ga, gb = operands(mx, M, N, K, INT8, INT8, 310)
    need = mx.mx_workspace_bytes("gemm", M, N, K, INT8, INT8)
    assert need >= (M + N) * K * 3
    want = mx.mx_gemm(ga[0], ga[1], INT8, gb[0], gb[1], INT8, K)
    ws = workspace(need)
    got = mx.mx_gemm_ws(ga[0], ga[1], INT8, gb[0], gb[1], INT8, K, ws[:need])
    assert bits_equal(got, want)
    with pytest.raises(mx.MxError) as err:
        mx.mx_gemm_ws(ga[0], ga[1], INT8, gb[0], gb[1], INT8, K, ws[:need - 1])
    assert err.value.status == mx.MX_ERR_WORKSPACE


def test_gemm_ws_without_scratch_needs_no_workspace(mx):
    M, N, K = 512, 512, 512
    _, ga, gb = operands(mx, M, N, K, FP8, FP4, 320)
    assert mx.mx_workspace_bytes("gemm", M, N, K, FP8, FP4) == 0
    want = mx.mx_gemm(ga[0], ga[1], FP8, gb[0], gb[1], FP4, K)
    assert bits_equal(mx.mx_gemm_ws(ga[0], ga[1], FP8, gb[0], gb[1], FP4, K, None), want)
    assert bits_equal(mx.mx_gemm_ws(ga[0], ga[1], FP8, gb[0], gb[1], FP4, K, workspace(16)), want)


Q_CASES = [
    ("ragged", 300, 520, 640, FP8, E2M3, E3M2, 0),           # Float32 C in scratch, then the row cast
    ("few_rows", 32, 2048, 1024, FP4, FP4, FP8, 1),
    ("tiled_trunc", 512, 512, 512, FP8, FP8, FP8, 2),        # toward zero is not cast in the epilogue
    ("int8_split", 4096, 4096, 1024, INT8, INT8, INT8, 0),   # Float32 C and the E2M3 halves side by side
]


@pytest.mark.parametrize("case", Q_CASES, ids=[c[0] for c in Q_CASES])
def test_gemm_q_ws_matches_pool_route(mx, case):
    _, M, N, K, fa, fb, fc, rnd = case
    _, ga, gb = operands(mx, M, N, K, fa, fb, 330)
    need = mx.mx_workspace_bytes("gemm_q", M, N, K, fa, fb)
    assert need >= M * N * 4
    want = mx.mx_gemm_q(ga[0], ga[1], fa, gb[0], gb[1], fb, K, fc, rnd)
    ws = workspace(need)
    got = mx.mx_gemm_q_ws(ga[0], ga[1], fa, gb[0], gb[1], fb, K, fc, rnd, ws[:need])
    assert bits_equal(got[0], want[0]) and bits_equal(got[1], want[1])
    with pytest.raises(mx.MxError) as err:
        mx.mx_gemm_q_ws(ga[0], ga[1], fa, gb[0], gb[1], fb, K, fc, rnd, ws[:need - 1])
    assert err.value.status == mx.MX_ERR_WORKSPACE


def test_epilogue_cast_ignores_the_workspace(mx):
    M, N, K = 2048, 2048, 1024                                # 64 whole tiles: the tiled kernel's route
    _, ga, gb = operands(mx, M, N, K, FP8, FP8, 340)
    want = mx.mx_gemm_q(ga[0], ga[1], FP8, gb[0], gb[1], FP8, K, FP8, 0)
    ws = workspace(mx.mx_workspace_bytes("gemm_q", M, N, K, FP8, FP8))
    got = mx.mx_gemm_q_ws(ga[0], ga[1], FP8, gb[0], gb[1], FP8, K, FP8, 0, ws)
    assert bits_equal(got[0], want[0]) and bits_equal(got[1], want[1])
    torch.cuda.synchronize()
    assert torch.all(ws == 0xA5)                              # C never existed at more than the format's width
