"""Stage 5 (Section 4, "Edge cases"): non-power-of-two dimensions.  The paper names
1023, 4097 and 1537; those leave rows unaligned to 16 bytes, which sends them to
the element-wise kernel.  Also here: the degenerate shapes of the operation
(one row, one column, empty batch), in-place operation, and misaligned bases."""
import numpy as np
import pytest
import torch

import gpu_harness as H
import compare
import oracle
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N", [(1023, 1023), (33, 4097), (129, 1537), (4097, 24), (1537, 1023),
                                 (5, 8193), (3, 40001), (65, 2049), (9, 16391), (7, 33001),
                                 (3, 131079), (2, 131080), (5, 65535), (3, 98305), (6, 7), (6, 9), (11, 3)])
def test_paper_edge_dims(gpu_device, M, N, dtype):
    H.check_case(inputs.random_case(5, 800 + 2 * dtype, M, N, dtype, 1e-6), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N", [(1, 1), (1, 8), (7, 1), (1, 8192), (2, 3), (1, 65), (5, 12)])
def test_degenerate_shapes(gpu_device, M, N, dtype):
    H.check_case(inputs.random_case(5, 820 + 2 * dtype, M, N, dtype, 1e-6), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
def test_empty_batch(gpu_device, dtype):
    x = torch.empty((0, 256), dtype=H.torch_dtype(dtype), device=gpu_device)
    w = torch.ones(256, dtype=H.torch_dtype(dtype), device=gpu_device)
    y = binding.rmsnorm_fwd(x, w, 1e-6)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (0, 256)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [4096, 13824, 1023])
def test_in_place(gpu_device, dtype, N):
    case = inputs.random_case(5, 840 + 2 * dtype, 97, N, dtype, 1e-6)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, dtype)
    wd = H.to_device(case["w"], dtype, gpu_device)
    for v in H.ALL_MODES:
        xd = H.to_device(case["x"], dtype, gpu_device)
        H.say(f"in place {case['name']} mode={H.mode_name(v)}")
        try:
            H.launch_mode(xd, wd, 1e-6, v, xd)
        except binding.RmsnormError as e:
            if e.status == binding.RMSNORM_ERR_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        compare.check_parity(H.to_host(xd, dtype), want, dtype, f"in place {v}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_misaligned_base_pointers(gpu_device, dtype):
    """An aligned N with bases one element off a 16-byte boundary: dispatch must fall back
    to the element-aligned kernel, stay inside the buffers and match the oracle; so must
    the element-wise kernel."""
    M, N = 41, 2048
    case = inputs.random_case(5, 860 + 2 * dtype, M, N, dtype, 1e-6)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, dtype)
    td = H.torch_dtype(dtype)
    xbuf = torch.zeros(M * N + 8, dtype=td, device=gpu_device)
    wbuf = torch.zeros(N + 8, dtype=td, device=gpu_device)
    xd = xbuf[1:1 + M * N].view(M, N)
    wd = wbuf[3:3 + N]
    xd.copy_(H.to_device(case["x"], dtype, gpu_device))
    wd.copy_(H.to_device(case["w"], dtype, gpu_device))
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1)
    assert binding.rmsnorm_select_variant(xd, wd, y) == binding.RMSNORM_VARIANT_UNALIGNED
    H.say(f"misaligned bases {inputs.DTYPE_NAMES[dtype]}")
    binding.rmsnorm_fwd(xd, wd, 1e-6, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype, offset_elems=1)
    compare.check_parity(H.to_host(y, dtype), want, dtype, "misaligned bases")
    whole2, y2 = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=3)
    binding.rmsnorm_fwd_variant(xd, wd, 1e-6, binding.RMSNORM_VARIANT_GENERIC, y2)
    torch.cuda.synchronize()
    assert H.guards_intact(whole2, M, N, dtype, offset_elems=3)
    compare.check_parity(H.to_host(y2, dtype), want, dtype, "misaligned bases, element-wise")
    # x and y at different offsets from a 16-byte boundary: no cut of the rows aligns both
    whole3, y3 = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=2)
    assert binding.rmsnorm_select_variant(xd, wd, y3) == binding.RMSNORM_VARIANT_UNALIGNED
    binding.rmsnorm_fwd(xd, wd, 1e-6, y3)
    torch.cuda.synchronize()
    assert H.guards_intact(whole3, M, N, dtype, offset_elems=2)
    compare.check_parity(H.to_host(y3, dtype), want, dtype, "misaligned bases, x and y skewed differently")
    for v in (binding.RMSNORM_VARIANT_WAVE, binding.RMSNORM_VARIANT_BLOCK,
              binding.RMSNORM_VARIANT_SUBWAVE) + \
            tuple(("threads", g) for g in H.THREADS):
        with pytest.raises(binding.RmsnormError) as e:
            H.launch_mode(xd, wd, 1e-6, v, y)
        assert e.value.status == binding.RMSNORM_ERR_UNSUPPORTED


def test_binding_rejects_mismatched_tensors(gpu_device):
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device=gpu_device)
    w = torch.ones(64, dtype=torch.bfloat16, device=gpu_device)
    with pytest.raises(ValueError):
        binding.rmsnorm_fwd(x, w[:32], 1e-6)
    with pytest.raises(ValueError):
        binding.rmsnorm_fwd(x, w.float(), 1e-6)
    with pytest.raises(ValueError):
        binding.rmsnorm_fwd(x.t(), w[:4], 1e-6)
    with pytest.raises(ValueError):
        binding.rmsnorm_fwd(x, w, 1e-6, torch.zeros((4, 32), dtype=torch.bfloat16, device=gpu_device))
    with pytest.raises(ValueError):
        binding.rmsnorm_fwd(x.cpu(), w, 1e-6)
    with pytest.raises(binding.RmsnormError):
        binding.rmsnorm_fwd(x, w, -1.0)


def test_non_default_stream(gpu_device):
    case = inputs.random_case(5, 880, 64, 4096, inputs.BF16, 1e-6)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, inputs.BF16)
    xd = H.to_device(case["x"], inputs.BF16, gpu_device)
    wd = H.to_device(case["w"], inputs.BF16, gpu_device)
    torch.cuda.synchronize()
    s = torch.cuda.Stream(device=gpu_device)
    with torch.cuda.stream(s):
        y = binding.rmsnorm_fwd(xd, wd, 1e-6)
    s.synchronize()
    compare.check_parity(H.to_host(y, inputs.BF16), want, inputs.BF16, "side stream")
