"""The automatic path picks narrower workgroups for batches of one to three rounds of resident
workgroups (the block-size axis of the paper's playbook, Section 3.3 tier 1, chosen per launch):
the result must not depend on that choice beyond the summation order, so every such batch is
compared with the oracle, and with the forced thread count that the query names, bit for bit."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu

CASES = [(inputs.BF16, 1536, 8192), (inputs.FP16, 2048, 8192), (inputs.FP16, 3072, 4096), (inputs.BF16, 1100, 4096),
         (inputs.BF16, 4096, 2048), (inputs.FP32, 2560, 2048), (inputs.FP32, 1537, 4096), (inputs.FP16, 1300, 6144)]


@pytest.mark.parametrize("dtype,M,N", CASES)
def test_batches_that_take_narrower_workgroups(gpu_device, dtype, M, N):
    g0 = binding.rmsnorm_auto_threads_per_row(N, dtype)
    g = binding.rmsnorm_auto_threads_for_batch(M, N, dtype)
    assert g in (128, 256) and g < g0, (g0, g)
    case = inputs.random_case(12, 2300 + N % 61, M, N, dtype, 1e-5)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-5, dtype, 0)
    xd = H.to_device(case["x"], dtype, gpu_device)
    wd = H.to_device(case["w"], dtype, gpu_device)
    H.say(f"batch dispatch {M}x{N} {inputs.DTYPE_NAMES[dtype]}: {g} threads instead of {g0}")
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
    binding.rmsnorm_fwd(xd, wd, 1e-5, y)
    forced = binding.rmsnorm_fwd_tuned(xd, wd, 1e-5, g)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype)
    got = H.to_host(y, dtype)
    compare.check_parity(got, want, dtype, f"batch dispatch {M}x{N}")
    assert np.array_equal(got, H.to_host(forced, dtype))
