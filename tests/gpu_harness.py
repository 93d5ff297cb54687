"""Shared plumbing of the GPU parity tests: upload, call the C ABI through the
binding, download, compare with the oracle.  No arithmetic of the method here.

Each GPU step prints (and flushes) the case it is about to run, so that a fault
on the device can be traced to a test, a shape, a dtype and a kernel variant.
"""
from __future__ import annotations

import sys

import numpy as np

import oracle
import compare
from paper_2603_21331_amd import binding, inputs

GUARD = 64            # guard elements on each side of y (a multiple of 16 bytes)
VARIANTS = (binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_WAVE,
            binding.RMSNORM_VARIANT_BLOCK, binding.RMSNORM_VARIANT_GENERIC,
            binding.RMSNORM_VARIANT_UNALIGNED, binding.RMSNORM_VARIANT_SUBWAVE,
            binding.RMSNORM_VARIANT_STREAM, binding.RMSNORM_VARIANT_PACKED,
            binding.RMSNORM_VARIANT_QUEUE)
THREADS = (8, 16, 32, 64, 128, 256, 512, 1024)
# A mode is a variant code (0..3) or ("threads", G): every way the ABI can be told to run.
ALL_MODES = VARIANTS + tuple(("threads", g) for g in THREADS)


def mode_name(mode) -> str:
    if isinstance(mode, tuple):
        return f"threads{mode[1]}"
    return binding.VARIANT_NAMES[mode]


def launch_mode(x_dev, w_dev, eps: float, mode, y):
    """One call through the binding in the given mode; raises RmsnormError on a status."""
    if isinstance(mode, tuple):
        return binding.rmsnorm_fwd_tuned(x_dev, w_dev, eps, mode[1], y)
    return binding.rmsnorm_fwd_variant(x_dev, w_dev, eps, mode, y)


def say(msg: str) -> None:
    print(f"[gpu] {msg}", file=sys.stderr, flush=True)


def torch_dtype(dtype: int):
    import torch
    return {inputs.FP32: torch.float32, inputs.FP16: torch.float16,
            inputs.BF16: torch.bfloat16}[dtype]


def to_device(a: np.ndarray, dtype: int, device):
    """Storage array (float32, or uint16 bit patterns) -> device tensor of the real dtype."""
    import torch
    a = np.ascontiguousarray(a)
    if dtype == inputs.FP32:
        return torch.from_numpy(a).to(device)
    return torch.from_numpy(a.view(np.int16)).to(device).view(torch_dtype(dtype))


def to_host(t, dtype: int) -> np.ndarray:
    import torch
    if dtype == inputs.FP32:
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def sentinel_bits(dtype: int) -> int:
    return 0x7FC0DEAD if dtype == inputs.FP32 else 0x7FCD   # NaN patterns


def alloc_guarded(M: int, N: int, dtype: int, device, offset_elems: int = 0):
    """A y buffer with sentinel-filled guard zones; returns (whole, view)."""
    import torch
    n = M * N
    whole_bits = torch.full((GUARD + offset_elems + n + GUARD,), 0, dtype=torch.int32
                            if dtype == inputs.FP32 else torch.int16, device=device)
    s = sentinel_bits(dtype)
    if dtype != inputs.FP32 and s >= 0x8000:
        s -= 0x10000
    whole_bits.fill_(s)
    whole = whole_bits.view(torch_dtype(dtype))
    lo = GUARD + offset_elems
    return whole, whole[lo:lo + n].view(M, N)


def guards_intact(whole, M: int, N: int, dtype: int, offset_elems: int = 0) -> bool:
    import torch
    bits = whole.view(torch.int32 if dtype == inputs.FP32 else torch.int16)
    s = sentinel_bits(dtype)
    if dtype != inputs.FP32 and s >= 0x8000:
        s -= 0x10000
    lo = GUARD + offset_elems
    head = bits[:lo]
    tail = bits[lo + M * N:]
    return bool((head == s).all().item() and (tail == s).all().item())


def run_variant(x_dev, w_dev, eps: float, dtype: int, mode, what: str):
    """Runs one mode into a guarded buffer; None if that kernel does not support the shape."""
    import torch
    M, N = x_dev.shape
    whole, y = alloc_guarded(M, N, dtype, x_dev.device)
    say(f"{what}: {inputs.DTYPE_NAMES[dtype]} {M}x{N} eps={eps} mode={mode_name(mode)}")
    try:
        launch_mode(x_dev, w_dev, eps, mode, y)
    except binding.RmsnormError as e:
        if e.status == binding.RMSNORM_ERR_UNSUPPORTED and mode != binding.RMSNORM_VARIANT_AUTO:
            return None
        raise
    torch.cuda.synchronize()
    assert guards_intact(whole, M, N, dtype), f"{what}: wrote outside y"
    return to_host(y, dtype)


def check_case(case: dict, device, variants=ALL_MODES, nthreads: int = 0, want=None) -> dict:
    """Runs every requested mode on one input case and compares with the oracle."""
    dtype, eps = case["dtype"], case["eps"]
    if want is None:
        want = oracle.rmsnorm_oracle(case["x"], case["w"], eps, dtype, nthreads)
    x_dev = to_device(case["x"], dtype, device)
    w_dev = to_device(case["w"], dtype, device)
    stats = {}
    ran = 0
    for v in variants:
        got = run_variant(x_dev, w_dev, eps, dtype, v, case["name"])
        if got is None:
            continue
        ran += 1
        stats[mode_name(v)] = compare.check_parity(
            got, want, dtype, f"{case['name']} [{mode_name(v)}]")
    assert ran >= 1, f"{case['name']}: no variant ran"
    return stats
