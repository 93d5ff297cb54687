"""More rows than the largest grid (Section 4, stage 2: "tiny, standard, large"): above 2^20
workgroups the register-resident kernels of RMSNorm, softmax and LayerNorm take rows blockIdx,
blockIdx + grid, ... in a loop, and only there does a workgroup see a second row (the two LDS
slots of its cross-wave reduction alternate, its row pointers advance by the grid).  Every
forced thread count, the element-addressed kernel in its one-workgroup-per-row form (fp32 rows
never take the walking form), the streaming kernel, the element-wise kernel, the LDS-staged
kernel and the automatic path run M = 2^20 + 77 short rows and are compared with the oracle
element by element.  The several-rows-per-wavefront kernel caps its grid at 2^24 workgroups:
one case goes past that as well."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
import test_layernorm_gpu as LN
import test_softmax_gpu as SM
from paper_2603_21331_amd import binding, inputs, layernorm, softmax

pytestmark = pytest.mark.gpu

M_BIG = (1 << 20) + 77
THREADS = tuple(("threads", g) for g in (64, 128, 256, 512, 1024))


@pytest.mark.parametrize("dtype,N", [(inputs.BF16, 64), (inputs.FP32, 32)])
def test_rmsnorm_more_rows_than_the_grid_limit(gpu_device, dtype, N):
    case = inputs.random_case(7, 2100 + dtype, M_BIG, N, dtype, 1e-6)
    modes = (binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_WAVE, binding.RMSNORM_VARIANT_BLOCK,
             binding.RMSNORM_VARIANT_GENERIC, binding.RMSNORM_VARIANT_UNALIGNED, binding.RMSNORM_VARIANT_STREAM,
             binding.RMSNORM_VARIANT_PACKED, binding.RMSNORM_VARIANT_SUBWAVE) + THREADS
    stats = H.check_case(case, gpu_device, variants=modes)
    assert len(stats) >= 11, sorted(stats)          # every thread count and variant ran (BLOCK needs longer rows)
    # the element-addressed kernel ran in its one-workgroup-per-row form, which strides beyond
    # the grid limit (rows this short never take the walking form)
    P = 1 << 20
    assert binding.load().rmsnorm_unaligned_walk_grid(P, P + (1 << 30), P + (1 << 31), M_BIG, N, dtype) == 0


@pytest.mark.parametrize("dtype,N", [(inputs.FP16, 64), (inputs.FP32, 32)])
def test_softmax_more_rows_than_the_grid_limit(gpu_device, dtype, N):
    case = inputs.softmax_case(7, 2110 + dtype, M_BIG, N, dtype)
    modes = (0, 1, 3, 4, 5, 6, 7) + tuple(("threads", g) for g in (64, 256, 512, 1024))
    stats = SM.check(case, gpu_device, modes=modes)
    assert len(stats) >= 10, sorted(stats)


@pytest.mark.parametrize("dtype,N", [(inputs.BF16, 64), (inputs.FP32, 32)])
def test_layernorm_more_rows_than_the_grid_limit(gpu_device, dtype, N):
    case = inputs.layernorm_case(7, 2120 + 4 * dtype, M_BIG, N, dtype)
    modes = (0, 1, 3, 4, 5, 6, 7) + tuple(("threads", g) for g in (64, 256, 512, 1024))
    stats = LN.check(case, gpu_device, modes=modes)
    assert len(stats) >= 10, sorted(stats)


def test_rmsnorm_rows_of_a_workgroup_do_not_leak_into_each_other_across_the_stride(gpu_device):
    """Rows blockIdx and blockIdx + 2^20 go through one workgroup one after the other: each
    must equal the one-row call on it, bit for bit, for every thread count."""
    N = 64
    case = inputs.random_case(7, 2130, M_BIG, N, inputs.FP16, 1e-6)
    xd = H.to_device(case["x"], inputs.FP16, gpu_device)
    wd = H.to_device(case["w"], inputs.FP16, gpu_device)
    for g in (64, 128, 256, 512, 1024):
        H.say(f"stride independence threads={g}")
        full = binding.rmsnorm_fwd_tuned(xd, wd, 1e-6, g)
        for i in (0, 76, (1 << 20) - 1, 1 << 20, (1 << 20) + 76):
            one = binding.rmsnorm_fwd_tuned(xd[i:i + 1], wd, 1e-6, g)
            assert torch.equal(one.view(torch.int16)[0], full.view(torch.int16)[i]), (g, i)


def test_subwave_kernel_past_its_grid_cap(gpu_device):
    """8 lanes per row and 8 rows per wavefront: 2^24 workgroups cover 2^27 rows, so 2^27 + 13
    rows of 8 fp32 values (4.3 GB) make the workgroups stride.  The input is one seeded block
    of 2^20 rows repeated; the oracle computes the block once, every repetition of the output
    must equal the first bit for bit, and the first, the last and the 13 rows past the last
    full repetition are compared with the oracle."""
    N, ROWS, REPS, EXTRA = 8, 1 << 20, 128, 13
    M = ROWS * REPS + EXTRA
    case = inputs.random_case(7, 2140, ROWS, N, inputs.FP32, 1e-6)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, inputs.FP32)
    block = H.to_device(case["x"], inputs.FP32, gpu_device)
    xd = torch.cat([block.repeat(REPS, 1), block[:EXTRA]])
    assert xd.shape[0] == M and M > (1 << 24) * 8
    wd = H.to_device(case["w"], inputs.FP32, gpu_device)
    H.say(f"subwave {M}x{N} fp32")
    y = binding.rmsnorm_fwd_variant(xd, wd, 1e-6, binding.RMSNORM_VARIANT_SUBWAVE)
    torch.cuda.synchronize()
    bits = y[:ROWS * REPS].view(torch.int32).view(REPS, ROWS * N)
    for k in range(1, REPS):
        assert torch.equal(bits[k], bits[0]), f"repetition {k} differs"
    compare.check_parity(y[:ROWS].cpu().numpy(), want, inputs.FP32, "subwave first block")
    compare.check_parity(y[ROWS * (REPS - 1):ROWS * REPS].cpu().numpy(), want, inputs.FP32, "subwave last block")
    compare.check_parity(y[ROWS * REPS:].cpu().numpy(), want[:EXTRA], inputs.FP32, "subwave tail")
