"""Rows that are a multiple of 16 bytes but not of the 128-byte cache line: the automatic paths of
RMSNorm, softmax and LayerNorm send them to the kernels written for rows that are not 16-byte
aligned (through LDS when short, the element-addressed register kernel beyond), because a
wavefront of the aligned kernels then straddles the lines.  Checked here: the choice that
rmsnorm_select_variant reports, parity of the automatic path with the oracle, and that its bits
are those of the forced variant; row lengths on both sides of every boundary of the rule."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import binding, inputs, layernorm, softmax

pytestmark = pytest.mark.gpu

EPS = 1e-5
PACKED, UNALIGNED = "packed", "unaligned"

# (dtype, M, N, what RMSNorm / softmax / LayerNorm take; None: the rule does not apply)
CASES = [
    (inputs.FP16, 301, 120, None, None, None),               # 240 bytes: below the rule
    (inputs.FP16, 301, 136, PACKED, PACKED, None),           # 272 bytes; LayerNorm starts at 1 KiB
    (inputs.BF16, 300, 520, PACKED, PACKED, PACKED),         # 1040 bytes
    (inputs.FP16, 259, 768, None, None, None),               # 1536 bytes: twelve whole lines
    (inputs.FP16, 259, 776, PACKED, UNALIGNED, PACKED),      # 1552 bytes: softmax leaves LDS at 1.5 KiB
    (inputs.FP16, 259, 904, PACKED, UNALIGNED, UNALIGNED),   # 1808 bytes: LayerNorm at 1.75 KiB
    (inputs.BF16, 257, 1032, UNALIGNED, UNALIGNED, UNALIGNED),   # 2064 bytes: RMSNorm at 2 KiB
    (inputs.FP32, 200, 260, PACKED, PACKED, PACKED),         # 1040 bytes of fp32
    (inputs.FP32, 130, 2052, UNALIGNED, UNALIGNED, UNALIGNED),
    (inputs.FP16, 129, 8184, UNALIGNED, UNALIGNED, UNALIGNED),   # 16368 bytes, one vector short of 16 KiB
    (inputs.BF16, 700, 8184, UNALIGNED, UNALIGNED, UNALIGNED),   # enough rows for the walking forms
    (inputs.FP16, 65, 16376, UNALIGNED, UNALIGNED, UNALIGNED),   # 32752 bytes
    (inputs.BF16, 33, 16392, UNALIGNED, UNALIGNED, None),        # 32784 bytes: past LayerNorm's 32 KiB
    (inputs.FP16, 300, 544, PACKED, PACKED, PACKED),             # 1088 bytes: whole half lines, short
    (inputs.FP16, 200, 2080, None, UNALIGNED, None),             # 4160 bytes: whole half lines; only softmax moves
    (inputs.BF16, 17, 32776, UNALIGNED, None, None),             # 65552 bytes: past softmax's 64 KiB
]
RMS_VARIANT = {PACKED: binding.RMSNORM_VARIANT_PACKED, UNALIGNED: binding.RMSNORM_VARIANT_UNALIGNED}
SM_VARIANT = {PACKED: softmax.SOFTMAX_VARIANT_PACKED, UNALIGNED: softmax.SOFTMAX_VARIANT_UNALIGNED}
LN_VARIANT = {PACKED: layernorm.LAYERNORM_VARIANT_PACKED, UNALIGNED: layernorm.LAYERNORM_VARIANT_UNALIGNED}
ALIGNED = (binding.RMSNORM_VARIANT_SUBWAVE, binding.RMSNORM_VARIANT_WAVE, binding.RMSNORM_VARIANT_BLOCK)


@pytest.mark.parametrize("dtype,M,N,rms,sm,ln", CASES)
def test_rmsnorm(gpu_device, dtype, M, N, rms, sm, ln):
    case = inputs.random_case(6, 2000 + N % 97, M, N, dtype, EPS)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], EPS, dtype, 0)
    xd, wd = H.to_device(case["x"], dtype, gpu_device), H.to_device(case["w"], dtype, gpu_device)
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
    chosen = binding.rmsnorm_select_variant(xd, wd, y)
    assert chosen == RMS_VARIANT[rms] if rms else chosen in ALIGNED, (N, chosen)
    H.say(f"off-line rows rmsnorm {inputs.DTYPE_NAMES[dtype]} {M}x{N} -> {rms}")
    binding.rmsnorm_fwd(xd, wd, EPS, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype)
    got = H.to_host(y, dtype)
    compare.check_parity(got, want, dtype, case["name"])
    if rms:
        forced = H.to_host(binding.rmsnorm_fwd_variant(xd, wd, EPS, RMS_VARIANT[rms]), dtype)
        assert np.array_equal(got, forced), "the automatic path did not run the variant it reports"


@pytest.mark.parametrize("dtype,M,N,rms,sm,ln", CASES)
def test_softmax(gpu_device, dtype, M, N, rms, sm, ln):
    case = inputs.softmax_case(6, 2100 + N % 97, M, N, dtype, 1.5)
    want = oracle.softmax_oracle(case["x"], dtype)
    xd = H.to_device(case["x"], dtype, gpu_device)
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
    H.say(f"off-line rows softmax {inputs.DTYPE_NAMES[dtype]} {M}x{N} -> {sm}")
    softmax.softmax_fwd(xd, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype)
    got = H.to_host(y, dtype)
    compare.check_softmax_parity(got, want, dtype, case["name"])
    takes_packed = softmax.softmax_auto_threads_per_row(N, dtype) == 1
    assert takes_packed == (sm == PACKED)
    if sm:
        forced = H.to_host(softmax.softmax_fwd_variant(xd, SM_VARIANT[sm]), dtype)
        assert np.array_equal(got, forced), "the automatic path did not run the variant the rule names"


@pytest.mark.parametrize("dtype,M,N,rms,sm,ln", CASES)
def test_layernorm(gpu_device, dtype, M, N, rms, sm, ln):
    case = inputs.layernorm_case(6, 2200 + N % 97, M, N, dtype, mean=0.4, std=1.3)
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], EPS, dtype, stats=True)
    f64 = lambda a: inputs.storage_to_f64(a, dtype)
    scale = compare.layernorm_scale(f64(case["x"]), f64(case["w"]), f64(case["b"]), mean, rstd)
    xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
    H.say(f"off-line rows layernorm {inputs.DTYPE_NAMES[dtype]} {M}x{N} -> {ln}")
    layernorm.layernorm_fwd(xd, wd, bd, EPS, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype)
    got = H.to_host(y, dtype)
    compare.check_layernorm_parity(got, want, scale, dtype, case["name"])
    takes_packed = layernorm.layernorm_auto_threads_per_row(N, dtype) == 1
    assert takes_packed == (ln == PACKED)
    if ln:
        forced = H.to_host(layernorm.layernorm_fwd_variant(xd, wd, bd, EPS, LN_VARIANT[ln]), dtype)
        assert np.array_equal(got, forced), "the automatic path did not run the variant the rule names"


@pytest.mark.parametrize("dtype,M,N", [(inputs.BF16, 300, 520), (inputs.FP16, 257, 1032), (inputs.FP16, 700, 8184)])
def test_in_place(gpu_device, dtype, M, N):
    """y == x through the automatic path on rows the rule moves: the bits of the out-of-place call."""
    case = inputs.layernorm_case(6, 2300 + N % 97, M, N, dtype, mean=0.2, std=1.1)
    xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
    H.say(f"off-line rows in place {inputs.DTYPE_NAMES[dtype]} {M}x{N}")
    for name, call in (("rmsnorm", lambda src, dst: binding.rmsnorm_fwd(src, wd, EPS, dst)),
                       ("softmax", lambda src, dst: softmax.softmax_fwd(src, dst)),
                       ("layernorm", lambda src, dst: layernorm.layernorm_fwd(src, wd, bd, EPS, dst))):
        want = H.to_host(call(xd, torch.empty_like(xd)), dtype)
        work = xd.clone()
        call(work, work)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_host(work, dtype), want), name
