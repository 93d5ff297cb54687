"""Inputs past 2^31 elements and 2^32 bytes, through the C ABI: every row offset in the kernels
must be 64-bit.  The input is one seeded block of 4096 rows repeated 74 times on the device
(303104 x 8192 of a 16-bit type: 2.48 G elements, 4.97 GB); the oracle computes the block once,
every repetition in the output must equal the first bit for bit (rows are independent), and the
first and the last repetition are compared with the oracle element by element."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import binding, crossentropy, inputs, layernorm, rowsum, softmax

pytestmark = pytest.mark.gpu

ROWS, N, REPS = 4096, 8192, 74


def tiled(block, dtype, device):
    xd = H.to_device(block, dtype, device).repeat(REPS, 1)
    assert xd.numel() > 2 ** 31 and xd.numel() * xd.element_size() > 2 ** 32
    return xd


def tiles_identical(y, per_row):
    bits = y.view(torch.int16 if y.dtype != torch.float32 else torch.int32).view(REPS, ROWS * per_row)
    return all(torch.equal(bits[k], bits[0]) for k in range(1, REPS))


def test_rmsnorm_past_4gib(gpu_device):
    case = inputs.random_case(9, 2000, ROWS, N, inputs.BF16, 1e-5)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], case["eps"], inputs.BF16)
    xd = tiled(case["x"], inputs.BF16, gpu_device)
    H.say(f"rmsnorm {tuple(xd.shape)} bf16")
    y = binding.rmsnorm_fwd(xd, H.to_device(case["w"], inputs.BF16, gpu_device), case["eps"])
    torch.cuda.synchronize()
    assert tiles_identical(y, N)
    for k in (0, REPS - 1):
        compare.check_parity(H.to_host(y[k * ROWS:(k + 1) * ROWS], inputs.BF16), want, inputs.BF16, f"rmsnorm tile {k}")


def test_layernorm_past_4gib(gpu_device):
    case = inputs.layernorm_case(9, 2004, ROWS, N, inputs.BF16)
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], case["eps"], inputs.BF16, stats=True)
    f64 = lambda a: inputs.storage_to_f64(a, inputs.BF16)
    scale = compare.layernorm_scale(f64(case["x"]), f64(case["w"]), f64(case["b"]), mean, rstd)
    xd = tiled(case["x"], inputs.BF16, gpu_device)
    H.say(f"layernorm {tuple(xd.shape)} bf16")
    y = layernorm.layernorm_fwd(xd, H.to_device(case["w"], inputs.BF16, gpu_device),
                                H.to_device(case["b"], inputs.BF16, gpu_device), case["eps"])
    torch.cuda.synchronize()
    assert tiles_identical(y, N)
    for k in (0, REPS - 1):
        compare.check_layernorm_parity(H.to_host(y[k * ROWS:(k + 1) * ROWS], inputs.BF16), want, scale, inputs.BF16,
                                       f"layernorm tile {k}")


def test_softmax_past_4gib(gpu_device):
    case = inputs.softmax_case(9, 2008, ROWS, N, inputs.FP16)
    want = oracle.softmax_oracle(case["x"], inputs.FP16)
    xd = tiled(case["x"], inputs.FP16, gpu_device)
    H.say(f"softmax {tuple(xd.shape)} fp16")
    y = softmax.softmax_fwd(xd)
    torch.cuda.synchronize()
    assert tiles_identical(y, N)
    for k in (0, REPS - 1):
        compare.check_softmax_parity(H.to_host(y[k * ROWS:(k + 1) * ROWS], inputs.FP16), want, inputs.FP16,
                                     f"softmax tile {k}")


def test_crossentropy_past_4gib(gpu_device):
    case = inputs.crossentropy_case(9, 2012, ROWS, N, inputs.FP16, 2.0)
    want = oracle.crossentropy_oracle(case["x"], case["target"], inputs.FP16)
    xd = tiled(case["x"], inputs.FP16, gpu_device)
    td = torch.from_numpy(case["target"]).to(gpu_device).repeat(REPS)
    H.say(f"crossentropy {tuple(xd.shape)} fp16")
    loss = crossentropy.crossentropy_fwd(xd, td)
    torch.cuda.synchronize()
    assert tiles_identical(loss, 1)
    for k in (0, REPS - 1):
        compare.check_crossentropy_parity(loss[k * ROWS:(k + 1) * ROWS].cpu().numpy(), want, f"crossentropy tile {k}")


def test_rowsum_past_4gib(gpu_device):
    case = inputs.rowsum_case(9, 2016, ROWS, N, inputs.FP16, 0.1, 1.0)
    want_y, want_abs = oracle.rowsum_oracle(case["x"], inputs.FP16, with_abs=True)
    xd = tiled(case["x"], inputs.FP16, gpu_device)
    H.say(f"rowsum {tuple(xd.shape)} fp16")
    y = rowsum.rowsum_fwd(xd)
    torch.cuda.synchronize()
    assert tiles_identical(y, 1)
    for k in (0, REPS - 1):
        compare.check_rowsum_parity(y[k * ROWS:(k + 1) * ROWS].cpu().numpy(), want_y, want_abs, N, f"rowsum tile {k}")
