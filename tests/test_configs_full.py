"""The benchmark workloads at their full sizes, every element against the oracle,
in the launch configuration bench.py times (automatic dispatch); the forced
variants run too wherever they support the shape."""
import pytest

import gpu_harness as H
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu


def test_config2_bf16_4096x4096(gpu_device):
    stats = H.check_case(inputs.config2(), gpu_device)
    H.say(f"cfg2 stats {stats}")


def test_config3_bf16_16384x8192_headline(gpu_device):
    case = inputs.config3()
    stats = H.check_case(case, gpu_device,
                         variants=(binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_WAVE,
                                   ("threads", 128), ("threads", 512), ("threads", 1024)))
    H.say(f"cfg3 stats {stats}")
    # sanity band, not the pass bar: fp32 accumulation should leave well under 1 % of the
    # outputs one bf16 ulp away from the fp64 oracle
    assert stats["auto"]["frac_off"] < 0.01


@pytest.mark.parametrize("N", inputs.CONFIG4_N)
def test_config4_fp16_shape_sweep(gpu_device, N):
    case = inputs.config4(N)
    assert case["M"] == 8191
    stats = H.check_case(case, gpu_device)
    H.say(f"cfg4 N={N} stats {stats}")
