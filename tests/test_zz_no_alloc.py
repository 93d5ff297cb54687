"""rmsnorm_fwd_static, the entry point that allocates nothing (its counters sit in a fixed block
of the library's static device array), against rmsnorm_fwd_workspace, the entry point it is a
variant of: called through the C ABI, two calls in a row on the one shared block, the second on
a smaller input, each compared bit for bit with the workspace entry point and within the stated
tolerance with the oracle.  Also: what it rejects, and that it is the library, not the caller,
that keeps the counters at zero between calls."""
import ctypes

import numpy as np
import pytest
import torch

import gpu_harness as H
import oracle
import compare
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu

EPS = 1e-5


def _raw_call(fn, xd, wd, yd, M, N, dtype, *extra):
    stream = torch.cuda.current_stream(xd.device).cuda_stream
    return fn(xd.data_ptr(), wd.data_ptr(), yd.data_ptr(), M, N, ctypes.c_float(EPS), dtype, stream, *extra)


def test_static_entry_matches_the_workspace_entry_on_two_calls_in_a_row(gpu_device):
    lib = binding.load()
    ws = binding.new_workspace(gpu_device)
    wbytes = ws.numel() * ws.element_size()
    # the second call is smaller in both dimensions (fewer rows, shorter rows, another chunk count)
    for M, N, dtype in ((3001, 8192, inputs.BF16), (777, 5120, inputs.BF16)):
        case = inputs.random_case(8, 1200 + N % 89, M, N, dtype, EPS)
        want = oracle.rmsnorm_oracle(case["x"], case["w"], EPS, dtype, 0)
        xd = H.to_device(case["x"], dtype, gpu_device)
        wd = H.to_device(case["w"], dtype, gpu_device)
        y_ws = torch.empty_like(xd)
        whole, y_st = H.alloc_guarded(M, N, dtype, gpu_device)
        H.say(f"no-alloc entry {M}x{N}: workspace entry")
        assert _raw_call(lib.rmsnorm_fwd_workspace, xd, wd, y_ws, M, N, dtype, ws.data_ptr(), wbytes) == binding.RMSNORM_OK
        H.say(f"no-alloc entry {M}x{N}: static entry")
        assert _raw_call(lib.rmsnorm_fwd_static, xd, wd, y_st, M, N, dtype) == binding.RMSNORM_OK
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype)
        got = H.to_host(y_st, dtype)
        assert np.array_equal(got, H.to_host(y_ws, dtype)), f"{M}x{N}: static and workspace entry points differ"
        compare.check_parity(got, want, dtype, f"static entry {M}x{N}")
    # a third call straight after, on the first size again, still finds its counters at zero
    case = inputs.random_case(8, 1290, 3001, 8192, inputs.BF16, EPS)
    xd = H.to_device(case["x"], inputs.BF16, gpu_device)
    wd = H.to_device(case["w"], inputs.BF16, gpu_device)
    a, b = torch.empty_like(xd), torch.empty_like(xd)
    H.say("no-alloc entry: third call")
    assert _raw_call(lib.rmsnorm_fwd_static, xd, wd, a, 3001, 8192, inputs.BF16) == binding.RMSNORM_OK
    assert _raw_call(lib.rmsnorm_fwd_workspace, xd, wd, b, 3001, 8192, inputs.BF16, ws.data_ptr(), wbytes) == binding.RMSNORM_OK
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_static_entry_rejects_what_its_fixed_scratch_does_not_cover(gpu_device):
    lib = binding.load()
    x = torch.zeros((2, 32776), dtype=torch.bfloat16, device=gpu_device)     # 4097 vectors per row
    w = torch.ones(32776, dtype=torch.bfloat16, device=gpu_device)
    y = torch.full_like(x, 5.0)
    assert _raw_call(lib.rmsnorm_fwd_static, x, w, y, 2, 32776, inputs.BF16) == binding.RMSNORM_ERR_TOO_LARGE
    # 2^30 rows: rejected on the row count alone, before any pointer is used
    assert _raw_call(lib.rmsnorm_fwd_static, x, w, y, 1 << 30, 8192, inputs.BF16) == binding.RMSNORM_ERR_TOO_LARGE
    # rows the kernel does not take for other reasons
    x2 = torch.zeros((2, 4096), dtype=torch.bfloat16, device=gpu_device)
    assert _raw_call(lib.rmsnorm_fwd_static, x2, w, y, 2, 4096, inputs.BF16) == binding.RMSNORM_ERR_UNSUPPORTED
    assert _raw_call(lib.rmsnorm_fwd_static, x2, w, y, 2, 4095, inputs.BF16) == binding.RMSNORM_ERR_UNSUPPORTED
    assert _raw_call(lib.rmsnorm_fwd_static, x2, w, y, -1, 8192, inputs.BF16) == binding.RMSNORM_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert bool((y == 5.0).all().item()), "a rejected call wrote to y"
    assert "larger" in binding.rmsnorm_status_string(binding.RMSNORM_ERR_TOO_LARGE)
