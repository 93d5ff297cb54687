"""A seeded random sweep of shapes, storage types and pointer offsets through the automatic
path of RMSNorm, softmax and LayerNorm, against the CPU oracle element by element: row lengths
from 1 to 20000 (log-uniform, so that every kernel family is hit), batches of 1 to 3000 rows
(capped so that the oracle stays fast), x, w, b and y each at its own offset of 0 to 70 elements
from a 256-byte boundary (so rows start anywhere relative to the 16-byte boundaries and the
128-byte lines, and y need not share x's offset), guard zones around y; and a second set whose
rows and offsets are all multiples of 16 bytes."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
import test_layernorm_gpu as LN
from paper_2603_21331_amd import binding, inputs, layernorm, softmax

pytestmark = pytest.mark.gpu

CASES = 48
ALIGNED_CASES = 36      # cases CASES .. CASES + ALIGNED_CASES - 1, see draw


def draw(k: int):
    rng = np.random.default_rng(7000 + k)
    dtype = [inputs.FP32, inputs.FP16, inputs.BF16][k % 3]
    if k >= CASES:
        # Rows and pointers that are multiples of 16 bytes, mostly not of the 128-byte line and
        # often not of its 64-byte halves: the vector kernels can take them, and the automatic
        # path decides by the lines which of them does.  All offsets a multiple of 16 bytes.
        per16 = 16 // inputs.DTYPE_BYTES[dtype]
        N = per16 * int(np.exp(rng.uniform(0.0, np.log(20000.0 / per16))))
        M = int(min(3000, max(1, rng.integers(1, 3001)), max(1, 3_000_000 // N)))
        offs = [per16 * int(o) for o in rng.integers(0, 9, size=4)]
        if k % 3 == 0:
            offs = [0, 0, 0, 0]
        return dtype, M, N, offs
    N = int(np.exp(rng.uniform(0.0, np.log(20000.0))))
    if k % 4 == 0:
        N = max(1, N // 8 * 8 + int(rng.integers(-1, 2)))     # next to a multiple of 16 bytes
    M = int(min(3000, max(1, rng.integers(1, 3001)), max(1, 3_000_000 // N)))
    offs = [int(o) for o in rng.integers(0, 71, size=4)]
    if k % 5 == 0:
        offs[3] = offs[0]                                       # y at x's offset
    return dtype, M, N, offs


def placed(a, dtype, device, off, shape):
    """The array on the device, `off` elements past a 256-byte boundary."""
    buf = torch.zeros(a.size + 128, dtype=H.torch_dtype(dtype), device=device)
    assert buf.data_ptr() % 256 == 0
    view = buf[off:off + a.size].view(*shape)
    view.copy_(H.to_device(a.reshape(shape), dtype, device))
    return view


@pytest.mark.parametrize("k", range(CASES + ALIGNED_CASES))
def test_random_shape_and_offsets(gpu_device, k):
    dtype, M, N, (ox, ow, ob, oy) = draw(k)
    case = inputs.layernorm_case(11, 2000 + 4 * k, M, N, dtype, 1e-5, mean=0.25, std=1.5)
    xd = placed(case["x"], dtype, gpu_device, ox, (M, N))
    wd = placed(case["w"], dtype, gpu_device, ow, (N,))
    bd = placed(case["b"], dtype, gpu_device, ob, (N,))
    name = f"random {k}: {inputs.DTYPE_NAMES[dtype]} {M}x{N} offsets {ox},{ow},{ob},{oy}"

    H.say(name + " rmsnorm")
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=oy)
    binding.rmsnorm_fwd(xd, wd, 1e-5, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype, offset_elems=oy), name
    compare.check_parity(H.to_host(y, dtype), oracle.rmsnorm_oracle(case["x"], case["w"], 1e-5, dtype), dtype,
                         name + " rmsnorm")

    H.say(name + " softmax")
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=oy)
    softmax.softmax_fwd(xd, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype, offset_elems=oy), name
    compare.check_softmax_parity(H.to_host(y, dtype), oracle.softmax_oracle(case["x"], dtype), dtype,
                                 name + " softmax")

    H.say(name + " layernorm")
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=oy)
    layernorm.layernorm_fwd(xd, wd, bd, 1e-5, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype, offset_elems=oy), name
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    compare.check_layernorm_parity(H.to_host(y, dtype), want, LN.scale_of(case, mean, rstd), dtype,
                                   name + " layernorm")
