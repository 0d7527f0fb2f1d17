"""The entry point that allocates nothing (srm_linear_argmax_noalloc) against the existing one
(srm_linear, epilogue 3, with a caller's scratch buffer), through the C ABI: two calls in a row,
the second on a smaller input, bit-exact (integer results)."""
import numpy as np
import pytest
import torch

import srm_synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def srm():
    import paper_2605_08696_amd as pkg
    pkg.lib()
    return pkg


def _case(srm, dtype, M, N, K, seed, with_bias):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32) if with_bias else None
    tt = torch.bfloat16 if dtype == srm.SRM_BF16 else torch.float32
    if dtype == srm.SRM_BF16:
        A, W = srm_synth.round_to_bf16(A), srm_synth.round_to_bf16(W)
    dA, dW = to_dev(A, tt), to_dev(W, tt)
    dB = None if bias is None else to_dev(bias)
    print(f"no-alloc argmax dtype={dtype} M={M} N={N} K={K} bias={with_bias}", flush=True)
    want = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    scratch = torch.empty(srm.linear_scratch_bytes(M, N), dtype=torch.uint8, device="cuda")
    srm.linear(dtype, 3, dA, dW, dB, out=None, argmax=want, scratch=scratch)
    got = torch.full((M,), -2, dtype=torch.int32, device="cuda")
    srm.linear_argmax_noalloc(dtype, dA, dW, dB, got)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), want.cpu().numpy())
    # and against the definition, on the kernel's own precision: fp64 product of the same operands
    ref = A.astype(np.float64) @ W.astype(np.float64).T + (0 if bias is None else bias)
    top = np.sort(ref, axis=1)
    clear = (top[:, -1] - top[:, -2]) > 1e-4 * np.abs(ref).max()
    np.testing.assert_array_equal(got.cpu().numpy()[clear], ref.argmax(axis=1)[clear])


@pytest.mark.parametrize("dtype_name", ["bf16", "fp32"])
def test_two_calls_in_a_row_the_second_smaller(srm, dtype_name):
    dtype = srm.SRM_BF16 if dtype_name == "bf16" else srm.SRM_FP32
    _case(srm, dtype, 700, 5000, 256, seed=1, with_bias=True)     # several row and column tiles, ragged edges
    _case(srm, dtype, 37, 130, 64, seed=2, with_bias=False)       # smaller: stale partials of the first call lie beyond
    _case(srm, dtype, 1, 64, 64, seed=3, with_bias=True)


def test_largest_shape_and_rejection(srm):
    cap = srm.linear_argmax_noalloc_max_bytes()
    assert cap == 8 << 20
    M, N, K = 2097, 32000, 64                                   # the largest row count at the LM head's width
    assert srm.linear_scratch_bytes(M, N) <= cap < srm.linear_scratch_bytes(M + 1, N)
    _case(srm, srm.SRM_BF16, M, N, K, seed=4, with_bias=False)
    A = torch.zeros((M + 1, K), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((N, K), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(M + 1, dtype=torch.int32, device="cuda")
    with pytest.raises(srm.SrmError) as e:
        srm.linear_argmax_noalloc(srm.SRM_BF16, A, W, None, out)
    assert e.value.code == -1 and "scratch" in str(e.value)
