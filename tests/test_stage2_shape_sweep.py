"""Stage 2 (Section 4, "Shape sweep"): about ten shapes times three dtypes, covering
tiny, standard, large, non-square and workload-specific sizes.  The paper prints the
sweep table for matmul only and says the other kernels have analogous ones; this is
the RMSNorm one: the paper's three RMSNorm result shapes (kernel performance table),
transformer hidden sizes, and sizes on both sides of each kernel's limits."""
import pytest

import gpu_harness as H
from paper_2603_21331_amd import inputs

pytestmark = pytest.mark.gpu

# (name, M, N): every N here keeps rows 16-byte aligned; stage 5 covers the others.
SWEEP = [
    ("tiny", 128, 128),
    ("one_vector", 70, 8),
    ("head_dim_64", 1031, 64),
    ("head_dim_128", 4099, 128),
    ("head_dim_256", 515, 256),
    ("short_ragged", 333, 200),
    ("small", 512, 512),
    ("ragged_last_chunk", 301, 1000),
    ("standard", 1024, 4096),
    ("hidden_5120", 515, 5120),
    ("wave_limit", 259, 8192),
    ("just_past_wave_limit", 130, 8200),
    ("mlp_11008", 200, 11008),
    ("tall", 8192, 1024),
    ("wide_32768", 67, 32768),
    ("block_limit_fp32", 9, 65536),
    ("block_limit_16bit", 5, 131072),
    ("past_every_register_kernel", 5, 131080),
    ("long_262144", 3, 262144),
]


@pytest.mark.parametrize("dtype", [inputs.FP32, inputs.FP16, inputs.BF16])
@pytest.mark.parametrize("name,M,N", SWEEP, ids=[s[0] for s in SWEEP])
def test_shape_sweep(gpu_device, name, M, N, dtype):
    case = inputs.random_case(1, 500 + 2 * dtype, M, N, dtype, 1e-6)
    H.check_case(case, gpu_device)


@pytest.mark.parametrize("which", [0, 1, 2])
def test_paper_result_shapes_fp16(gpu_device, which):
    """The three RMSNorm rows of the paper's kernel performance table, in its precision, on
    the inputs the benchmark's --all-configs leg times."""
    case = inputs.rmsnorm_paper_shape(which)
    assert (case["M"], case["N"]) == inputs.RMSNORM_PAPER_SHAPES[which] and case["dtype"] == inputs.FP16
    H.check_case(case, gpu_device)
