"""The automatic path at every aligned row length up to 8192 elements (every multiple of one
16-byte vector: all dispatch boundaries between lane groups, one wavefront per row, workgroups
of 256, 512 and 1024 threads, the resident and the LDS-staged kernels) and at odd lengths
beyond the LDS-staged kernel's 1024 elements, all five operations, all three dtypes, each
output compared with the CPU oracle element by element."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
import test_layernorm_gpu as LN
from paper_2603_21331_amd import binding, inputs, layernorm, softmax
from paper_2603_21331_amd import crossentropy as ce, rowsum as rs

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]
M = 19


def lengths(dtype):
    vec = 16 // inputs.DTYPE_BYTES[dtype]
    aligned = [vec * k for k in range(1, 8192 // vec + 1)]
    odd = list(range(1025, 9000, 97))
    return aligned[::1 if dtype != inputs.FP32 else 2] + odd      # about 1100 lengths per dtype


@pytest.mark.parametrize("dtype", DTYPES)
def test_rmsnorm_softmax_layernorm_every_length(gpu_device, dtype):
    for N in lengths(dtype):
        case = inputs.layernorm_case(8, 1200 + 4 * dtype, M, N, dtype, 1e-5, mean=0.5, std=1.5)
        xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
        H.say(f"every length: rmsnorm, softmax, layernorm {inputs.DTYPE_NAMES[dtype]} N={N}")
        wr, yr = H.alloc_guarded(M, N, dtype, gpu_device)
        ws, ys = H.alloc_guarded(M, N, dtype, gpu_device)
        wl, yl = H.alloc_guarded(M, N, dtype, gpu_device)
        binding.rmsnorm_fwd(xd, wd, 1e-5, yr)
        softmax.softmax_fwd(xd, ys)
        layernorm.layernorm_fwd(xd, wd, bd, 1e-5, yl)
        torch.cuda.synchronize()
        for whole in (wr, ws, wl):
            assert H.guards_intact(whole, M, N, dtype), f"N={N}: wrote outside an output"
        compare.check_parity(H.to_host(yr, dtype), oracle.rmsnorm_oracle(case["x"], case["w"], 1e-5, dtype),
                             dtype, f"rmsnorm N={N}")
        compare.check_softmax_parity(H.to_host(ys, dtype), oracle.softmax_oracle(case["x"], dtype), dtype,
                                     f"softmax N={N}")
        want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
        compare.check_layernorm_parity(H.to_host(yl, dtype), want, LN.scale_of(case, mean, rstd), dtype,
                                       f"layernorm N={N}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_crossentropy_rowsum_every_length(gpu_device, dtype):
    for N in lengths(dtype):
        case = inputs.crossentropy_case(8, 1220 + 4 * dtype, M, N, dtype, 2.0, ignore_every=9)
        t = np.asarray(case["target"], dtype=np.int64)
        xd = H.to_device(case["x"], dtype, gpu_device)
        td = torch.from_numpy(t).to(gpu_device)
        H.say(f"every length: cross-entropy, row sum {inputs.DTYPE_NAMES[dtype]} N={N}")
        loss = ce.crossentropy_fwd(xd, td)
        total = rs.rowsum_fwd(xd)
        torch.cuda.synchronize()
        compare.check_crossentropy_parity(loss.cpu().numpy(), oracle.crossentropy_oracle(case["x"], t, dtype),
                                          f"cross-entropy N={N}", exact_zero=(t < 0) | (t >= N))
        want_sum, want_abs = oracle.rowsum_oracle(case["x"], dtype, with_abs=True)
        compare.check_rowsum_parity(total.cpu().numpy(), want_sum, want_abs, N, f"row sum N={N}")
