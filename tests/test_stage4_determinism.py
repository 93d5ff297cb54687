"""Stage 4 (Section 4, "Determinism"): same input, repeated runs, bitwise identical
outputs.  The paper runs three times; here every variant runs three times into
the same buffer and twice into fresh buffers."""
import numpy as np
import pytest
import torch

import gpu_harness as H
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _bits(t, dtype):
    return H.to_host(t, dtype).copy()


def _repeat(case, device):
    dtype, eps = case["dtype"], case["eps"]
    xd = H.to_device(case["x"], dtype, device)
    wd = H.to_device(case["w"], dtype, device)
    for v in H.ALL_MODES:
        H.say(f"determinism {case['name']} mode={H.mode_name(v)}")
        y = torch.empty_like(xd)
        try:
            H.launch_mode(xd, wd, eps, v, y)
        except binding.RmsnormError as e:
            if e.status == binding.RMSNORM_ERR_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        first = _bits(y, dtype)
        for _ in range(2):
            H.launch_mode(xd, wd, eps, v, y)
            torch.cuda.synchronize()
            assert np.array_equal(_bits(y, dtype), first)
        for _ in range(2):
            fresh = torch.empty_like(xd)
            H.launch_mode(xd, wd, eps, v, fresh)
            torch.cuda.synchronize()
            assert np.array_equal(_bits(fresh, dtype), first)


def test_determinism_config5(gpu_device):
    _repeat(inputs.config5(), gpu_device)


@pytest.mark.parametrize("dtype", [inputs.FP32, inputs.BF16])
def test_determinism_other_dtypes(gpu_device, dtype):
    _repeat(inputs.random_case(4, 700 + 2 * dtype, 777, 5120, dtype, 1e-5), gpu_device)


@pytest.mark.parametrize("N", [4096, 128])
def test_rows_do_not_depend_on_their_neighbours(gpu_device, N):
    """Row i of a large call equals the one-row call on that row, bit for bit, within a
    variant: the grid shape must not leak into the arithmetic."""
    case = inputs.random_case(4, 710, 300, N, inputs.BF16, 1e-6)
    xd = H.to_device(case["x"], inputs.BF16, gpu_device)
    wd = H.to_device(case["w"], inputs.BF16, gpu_device)
    ran = 0
    for v in H.ALL_MODES[1:]:
        H.say(f"row independence N={N} mode={H.mode_name(v)}")
        try:
            full = H.to_host(H.launch_mode(xd, wd, 1e-6, v, None), inputs.BF16)
        except binding.RmsnormError as e:
            if e.status == binding.RMSNORM_ERR_UNSUPPORTED:
                continue
            raise
        ran += 1
        for i in (0, 3, 157, 299):
            one = H.to_host(H.launch_mode(xd[i:i + 1], wd, 1e-6, v, None), inputs.BF16)
            assert np.array_equal(one[0], full[i])
    assert ran >= 4
