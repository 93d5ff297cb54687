"""Stage 1 of the paper's five-stage correctness pipeline (Section 4, "Smoke
test"): one small input, every dtype, against the oracle at the tight tolerance."""
import pytest

import gpu_harness as H
from paper_2603_21331_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [inputs.FP32, inputs.FP16, inputs.BF16])
def test_smoke_128x128(gpu_device, dtype):
    case = inputs.random_case(0, 400 + 2 * dtype, 128, 128, dtype, 1e-6)
    H.check_case(case, gpu_device)


def test_config1_fp32_64x1024(gpu_device):
    H.check_case(inputs.config1(), gpu_device)
