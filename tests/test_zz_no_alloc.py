"""mx_gemm_qa_noalloc -- the entry point for callers that cannot allocate -- against mx_gemm_qa:
the same bytes, on two calls in a row that share the library's static scratch array, the second
with a smaller input (so stale contents of the first call lie behind what the second one writes)."""
import numpy as np
import pytest
import torch

from gpu_util import to_dev
from paper_2310_10537_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mx():
    from paper_2310_10537_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()
    return binding


def pair(mx, M, N, K, fa, fb, rnd, dt, seed):
    a = to_dev(inputs.student_t_bf16((M, K), seed=seed))
    gb = mx.mx_quantize(to_dev(inputs.gaussian_f32((N, K), seed=seed + 1, std=0.02)), 1, fb)
    want = mx.mx_gemm_qa(a, fa, rnd, gb[0], gb[1], fb, dtype=dt)
    out = torch.full((M, N), 7.0, dtype=dt, device="cuda")
    got = mx.mx_gemm_qa_noalloc(a, fa, rnd, gb[0], gb[1], fb, out)
    torch.cuda.synchronize()
    # A first launch may make the runtime load a code object; a repeat must not take anything from the
    # device.  (Free memory may still GROW meanwhile: pool memory of earlier work is returned lazily.)
    free_before = torch.cuda.mem_get_info()[0]
    mx.mx_gemm_qa_noalloc(a, fa, rnd, gb[0], gb[1], fb, out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before
    assert torch.equal(got.view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                       want.view(torch.int16 if dt == torch.bfloat16 else torch.int32)), (M, N, K, fa, fb)


@pytest.mark.parametrize("fa,fb,rnd", [(0, 0, 0), (2, 4, 1), (4, 1, 2)], ids=["e4m3", "e3m2xe2m1_away", "e2m1xe5m2_trunc"])
def test_two_calls_in_a_row_second_smaller(mx, fa, fb, rnd):
    # tiled route (32 whole tiles), then a smaller ragged problem on the shared-K / direct kernels
    pair(mx, 2048, 1024, 1024, fa, fb, rnd, torch.bfloat16, 900)
    pair(mx, 200, 136, 288, fa, fb, rnd, torch.float32, 902)
    pair(mx, 1, 64, 32, fa, fb, rnd, torch.float32, 904)


def test_full_size_and_limits(mx):
    # the 8192 x 4096 activation tensor of the transformer projection fits the static array
    pair(mx, 8192, 4096, 4096, 0, 0, 0, torch.bfloat16, 906)
    a = torch.zeros((8192 + 1024, 4096), dtype=torch.bfloat16, device="cuda")
    gb = mx.mx_quantize(torch.zeros((256, 4096), dtype=torch.float32, device="cuda"), 1, 0)
    out = torch.full((a.shape[0], 256), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(mx.MxError) as err:
        mx.mx_gemm_qa_noalloc(a, 0, 0, gb[0], gb[1], 0, out)
    assert err.value.status == mx.MX_ERR_TOO_LARGE and "scratch" in str(err.value)
    assert torch.all(out == 7.0)                                  # nothing was launched
    gi = mx.mx_quantize(torch.zeros((256, 4096), dtype=torch.float32, device="cuda"), 1, 5)
    with pytest.raises(mx.MxError) as err:
        mx.mx_gemm_qa_noalloc(a[:256], 5, 0, gi[0], gi[1], 5, out[:256])
    assert err.value.status == 5
    # zero-sized problems are no-ops
    mx.mx_gemm_qa_noalloc(a[:0], 0, 0, gb[0], gb[1], 0, out[:0])
