"""The entry points only enqueue kernels (no allocation, no copy, no synchronisation), so a
caller may record them into a HIP graph and replay it: the launch-bound small shapes
(configuration 1 is 3 microseconds of GPU time per call) are where that pays.  Each test
captures one call per operation on a side stream, replays the graph several times with new
input values written into the same buffers between replays (and the program's own eager work
and synchronisations in between), and checks every replay bit for bit against the eager call."""
import numpy as np
import pytest
import torch

import gpu_harness as H
from paper_2603_21331_amd import binding, crossentropy, inputs, layernorm, rowsum, softmax

pytestmark = pytest.mark.gpu

SHAPES = [(64, 1024, inputs.FP32), (333, 200, inputs.FP16), (257, 77, inputs.BF16),
          (128, 8192, inputs.BF16), (37, 40001, inputs.FP16)]


@pytest.mark.parametrize("M,N,dtype", SHAPES)
def test_all_five_operations_replay_from_a_graph(gpu_device, M, N, dtype):
    td = H.torch_dtype(dtype)
    gen = torch.Generator(device=gpu_device).manual_seed(1234 + N)

    def fresh():
        return (torch.randn((M, N), generator=gen, device=gpu_device, dtype=torch.float32) * 2.0).to(td)

    x = fresh()
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(td)
    b = (0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(td)
    t = torch.randint(0, N, (M,), generator=gen, device=gpu_device, dtype=torch.int64)
    outs = dict(rms=torch.empty_like(x), sm=torch.empty_like(x), ln=torch.empty_like(x),
                ce=torch.empty(M, dtype=torch.float32, device=gpu_device),
                lse=torch.empty(M, dtype=torch.float32, device=gpu_device),
                rs=torch.empty(M, dtype=torch.float32, device=gpu_device))

    def enqueue(o):
        binding.rmsnorm_fwd(x, w, 1e-6, o["rms"])
        softmax.softmax_fwd(x, o["sm"])
        layernorm.layernorm_fwd(x, w, b, 1e-5, o["ln"])
        crossentropy.crossentropy_fwd(x, t, o["ce"], o["lse"])
        rowsum.rowsum_fwd(x, o["rs"])

    enqueue(outs)                                   # eager warm-up: loads the libraries
    torch.cuda.synchronize()
    H.say(f"graph capture {M}x{N} {inputs.DTYPE_NAMES[dtype]}")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(outs)
    torch.cuda.synchronize()

    eager = {k: torch.empty_like(v) for k, v in outs.items()}
    for replay in range(3):
        x.copy_(fresh())                            # new values, same buffers
        t.copy_(torch.randint(0, N, (M,), generator=gen, device=gpu_device, dtype=torch.int64))
        for v in outs.values():
            v.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        enqueue(eager)
        torch.cuda.synchronize()
        for k in outs:
            got = outs[k].view(torch.uint8).cpu().numpy()
            want = eager[k].view(torch.uint8).cpu().numpy()
            assert np.array_equal(got, want), f"replay {replay}: {k} differs from the eager call"
