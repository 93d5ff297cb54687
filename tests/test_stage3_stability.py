"""Stage 3 (Section 4, "Numerical stability"): adversarial magnitudes.  For a
normalisation the paper names near-zero variance; added here are the overflow
and underflow ends of each storage type and rows dominated by one element."""
import numpy as np
import pytest

import gpu_harness as H
import oracle
from paper_2603_21331_amd import inputs

pytestmark = pytest.mark.gpu


def _case(name, x64, dtype, eps=1e-6, w64=None, seed=3):
    M, N = x64.shape
    w = inputs.normal_matrix(seed, 601, 1, N, dtype, 1.0, 0.1)[0] if w64 is None \
        else inputs.to_storage(w64, dtype)
    return dict(name=name, dtype=dtype, M=M, N=N, eps=eps, x=inputs.to_storage(x64, dtype), w=w)


@pytest.mark.parametrize("dtype", [inputs.FP32, inputs.FP16, inputs.BF16])
def test_near_zero_rows(gpu_device, dtype):
    """Rows that are exactly zero, almost zero, and constant (zero variance)."""
    N = 2048
    z = inputs.normal(3, 600, 0, 8 * N).reshape(8, N)
    tiny = {inputs.FP32: 1e-30, inputs.FP16: 1e-7, inputs.BF16: 1e-30}[dtype]
    z[0] = 0.0
    z[1] *= tiny
    z[2] = 0.75
    z[3] = -tiny
    z[4, 1:] = 0.0
    z[5] *= 1e-3
    z[6] = np.where(np.arange(N) % 2 == 0, 1.0, -1.0)
    case = _case("near_zero", z, dtype)
    H.check_case(case, gpu_device)
    # the all-zero row must come out as exact zeros from every variant
    want = oracle.rmsnorm_oracle(case["x"], case["w"], case["eps"], dtype)
    assert np.all(oracle.decode(want[0], dtype) == 0.0)


@pytest.mark.parametrize("dtype", [inputs.FP32, inputs.FP16, inputs.BF16])
def test_large_magnitudes(gpu_device, dtype):
    """Values near the top of the range whose squares still sum below FLT_MAX."""
    N = 4096
    z = inputs.normal(3, 602, 0, 6 * N).reshape(6, N)
    big = {inputs.FP32: 1e17, inputs.FP16: 2e4, inputs.BF16: 1e17}[dtype]
    z[0] *= big
    z[1] = np.clip(z[1] * big, -3 * big, 3 * big)
    z[2] = big
    z[3] *= 1e-3
    z[3, 77] = big
    z[4] *= big
    z[4, ::2] *= 1e-20 if dtype != inputs.FP16 else 1e-6
    H.check_case(_case("large_magnitudes", z, dtype), gpu_device)


def test_config5_fp16_adversarial(gpu_device):
    """Row scales 10^U(-4,4), 1 % zero rows, 1 % rows with one +/-60000 spike."""
    case = inputs.config5()
    assert len(case["zero_rows"]) == 41 and len(case["spike_rows"]) == 41
    assert not set(case["zero_rows"]) & set(case["spike_rows"])
    stats = H.check_case(case, gpu_device)
    H.say(f"cfg5 stats {stats}")


@pytest.mark.parametrize("dtype", [inputs.FP16, inputs.BF16])
def test_subnormal_outputs_are_not_flushed(gpu_device, dtype):
    """One dominant element pushes the rest of the row's outputs into the subnormal range."""
    N = 1024
    z = inputs.normal(3, 604, 0, 4 * N).reshape(4, N)
    small = {inputs.FP16: 3e-4, inputs.BF16: 1e-36}[dtype]
    huge = {inputs.FP16: 6e4, inputs.BF16: 1e3}[dtype]
    z *= small
    z[:, 5] = huge
    case = _case("subnormal_outputs", z, dtype, eps=0.0)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 0.0, dtype)
    mag = want & 0x7FFF
    sub = (mag != 0) & (mag < (0x0400 if dtype == inputs.FP16 else 0x0080))
    assert sub.sum() > 100, "the case must actually produce subnormal outputs"
    H.check_case(case, gpu_device, want=want)


def test_nan_and_inf_propagate(gpu_device):
    """Not part of the graded workloads: only the NaN positions are compared."""
    N = 512
    z = inputs.normal(3, 606, 0, 3 * N).reshape(3, N)
    x = inputs.to_storage(z, inputs.FP32)
    x[1, 7] = np.nan
    x[2, 9] = np.inf
    case = dict(name="nan_inf", dtype=inputs.FP32, M=3, N=N, eps=1e-6, x=x,
                w=inputs.normal_matrix(3, 607, 1, N, inputs.FP32, 1.0, 0.1)[0])
    want = oracle.rmsnorm_oracle(x, case["w"], 1e-6, inputs.FP32)
    xd = H.to_device(x, inputs.FP32, gpu_device)
    wd = H.to_device(case["w"], inputs.FP32, gpu_device)
    for v in H.ALL_MODES:
        got = H.run_variant(xd, wd, 1e-6, inputs.FP32, v, "nan_inf")
        if got is None:
            continue
        assert np.array_equal(np.isnan(got), np.isnan(want))
        assert np.array_equal(got[0], got[0]) and not np.isnan(got[0]).any()
