"""The work-queue form of LayerNorm's resident kernel (LAYERNORM_VARIANT_QUEUE): resident
workgroups of 256 or 512 threads plus one wavefront that draws their rows from counters in
device memory.  Checked here: parity with the oracle and the bits of the resident kernel on
every chunk count it is built for, batches around every boundary of the row bookkeeping, with
and without bias, in place, repeated launches (the counters must come back to zero: a launch on
counters that were left non-zero would skip rows, which a pre-filled y shows), the automatic
path at sizes where it takes this kernel, on two streams at once, and a call under graph
capture, which must take another kernel."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import inputs, layernorm

pytestmark = pytest.mark.gpu

EPS = 1e-5
Q = layernorm.LAYERNORM_VARIANT_QUEUE
CODES = {inputs.FP32: layernorm.LAYERNORM_DTYPE_FP32, inputs.FP16: layernorm.LAYERNORM_DTYPE_FP16,
         inputs.BF16: layernorm.LAYERNORM_DTYPE_BF16}


def _scale(case, mean, rstd):
    dtype = case["dtype"]
    return compare.layernorm_scale(inputs.storage_to_f64(case["x"], dtype), inputs.storage_to_f64(case["w"], dtype),
                                   None if case["b"] is None else inputs.storage_to_f64(case["b"], dtype), mean, rstd)


def _check(case, device, threads):
    dtype = case["dtype"]
    M, N = case["x"].shape
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], EPS, dtype, stats=True)
    xd = H.to_device(case["x"], dtype, device)
    wd = H.to_device(case["w"], dtype, device)
    bd = None if case["b"] is None else H.to_device(case["b"], dtype, device)
    # Same threads and chunks as the resident kernel, so the same bits, except where a thread holds
    # more than 24 elements: the resident kernel does not take those rows.
    elems = -(-N * inputs.DTYPE_BYTES[dtype] // 16 // threads) * (16 // inputs.DTYPE_BYTES[dtype])
    resident = H.to_host(layernorm.layernorm_fwd_tuned(xd, wd, bd, EPS, threads), dtype) if elems <= 24 else None
    first = None
    for rep in range(2):
        H.say(f"layernorm queue {case['name']} bias={bd is not None} rep={rep}")
        whole, y = H.alloc_guarded(M, N, dtype, device)
        layernorm.layernorm_fwd_variant(xd, wd, bd, EPS, Q, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype), f"{case['name']}: wrote outside y"
        got = H.to_host(y, dtype)
        compare.check_layernorm_parity(got, want, _scale(case, mean, rstd), dtype, f"{case['name']} [queue]")
        if resident is not None:
            assert np.array_equal(got, resident), f"{case['name']}: bits differ from the resident kernel"
        first = got if first is None else first
        assert np.array_equal(got, first), f"{case['name']}: bits differ from run to run"


# (dtype, N, threads that hold the row): every chunk count of either workgroup size, exact and
# ragged last chunks
SHAPES = [
    (inputs.FP16, 1600, 256),     # 200 vectors: one chunk, ragged
    (inputs.BF16, 2048, 256),     # 256 vectors: one full chunk
    (inputs.FP16, 3072, 256),     # 384 vectors: two chunks, ragged
    (inputs.FP16, 4096, 256),     # 512 vectors: two full chunks
    (inputs.FP16, 5120, 256),     # 640 vectors: three chunks, ragged (a shape of the paper's table)
    (inputs.BF16, 6144, 256),     # 768 vectors: three full chunks
    (inputs.FP16, 7168, 256),     # 896 vectors: four chunks, ragged; weight and bias stay packed
    (inputs.BF16, 8192, 256),     # 1024 vectors: four full chunks, packed weight and bias
    (inputs.FP16, 10248, 512),    # 1281 vectors: three chunks of 512, ragged
    (inputs.BF16, 12288, 512),    # 1536 vectors: three full chunks
    (inputs.BF16, 14336, 512),    # 1792 vectors: four chunks, ragged, packed weight and bias
    (inputs.FP16, 16384, 512),    # 2048 vectors: four full chunks, packed weight and bias
    (inputs.FP32, 512, 256),      # 128 vectors of fp32
    (inputs.FP32, 2048, 256),     # 512 vectors: two chunks
    (inputs.FP32, 3076, 256),     # 769 vectors: four chunks, ragged
    (inputs.FP32, 4096, 256),     # 1024 vectors: four full chunks
    (inputs.FP32, 5120, 512),     # 1280 vectors: three chunks of 512
    (inputs.FP32, 8192, 512),     # 2048 vectors: four full chunks
]


@pytest.mark.parametrize("dtype,N,threads", SHAPES)
def test_parity_and_bits_on_every_chunk_count(gpu_device, dtype, N, threads):
    takes, g, grid, shards, block_rows = layernorm.layernorm_queue_plan(1000, N, CODES[dtype])
    assert g == threads and grid % shards == 0 and not takes
    for k, M in enumerate((301, 2 * grid + 37)):
        case = inputs.layernorm_case(6, 1700 + N % 89, M, N, dtype, mean=0.3, std=1.2, bias=(k == 0))
        _check(case, gpu_device, threads)


@pytest.mark.parametrize("dtype,N,threads", [(inputs.FP16, 4096, 256), (inputs.BF16, 12288, 512)])
def test_row_bookkeeping(gpu_device, dtype, N, threads):
    """Batches below, at and past one and two rounds of the grid, fewer rows than shards, and
    batches that end inside a block of rows."""
    _, _, grid, shards, block_rows = layernorm.layernorm_queue_plan(1000, N, CODES[dtype])
    for k, M in enumerate((1, 2, shards - 1, shards * block_rows + 1, grid - 1, grid, grid + 1, 2 * grid,
                           2 * grid + block_rows - 1, 3 * grid + grid // 2 + 5)):
        case = inputs.layernorm_case(6, 1720 + 4 * dtype, M, N, dtype, mean=-0.2, std=1.3, bias=(k % 3 != 1))
        _check(case, gpu_device, threads)


def test_in_place_and_repeated_runs_are_bit_identical(gpu_device):
    dtype = inputs.FP16
    case = inputs.layernorm_case(6, 1740, 3000, 5120, dtype)
    xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
    first = H.to_host(layernorm.layernorm_fwd_variant(xd, wd, bd, EPS, Q), dtype)
    y = torch.empty_like(xd)
    for k in range(4):
        H.say(f"layernorm queue repeat {k}")
        y.fill_(7.0)
        layernorm.layernorm_fwd_variant(xd, wd, bd, EPS, Q, y)
        assert np.array_equal(H.to_host(y, dtype), first)
    H.say("layernorm queue in place")
    layernorm.layernorm_fwd_variant(xd, wd, bd, EPS, Q, xd)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(xd, dtype), first)


def test_rows_the_kernel_does_not_take(gpu_device):
    for dtype, N in ((inputs.FP16, 16392), (inputs.FP16, 4100), (inputs.FP32, 8196), (inputs.BF16, 65536)):
        case = inputs.layernorm_case(6, 1750, 4, N, dtype)
        xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
        with pytest.raises(layernorm.LayerNormError) as e:
            layernorm.layernorm_fwd_variant(xd, wd, bd, EPS, Q)
        assert e.value.status == layernorm.LAYERNORM_ERR_UNSUPPORTED, (dtype, N)


@pytest.mark.parametrize("dtype,M,N,threads", [(inputs.FP16, 16384, 4096, 256), (inputs.BF16, 4096, 12288, 512),
                                               (inputs.BF16, 12288, 8192, 0), (inputs.FP16, 3072, 16384, 0)])
def test_automatic_path_takes_the_queue_for_large_launches(gpu_device, dtype, M, N, threads):
    """128 MiB of 8 KiB rows, 96 MiB of 24 KiB rows, 192 MiB of 16 KiB rows and 96 MiB of 32 KiB rows:
    layernorm_fwd runs the work-queue kernel on the stream's own counters (default stream, a side
    stream, several times in a row) with the bits of the resident kernel (threads == 0: rows the
    resident kernel does not take in that shape; the forced variant stands in); one row less and
    the plan says it does not.  Sampled rows against the oracle."""
    code = CODES[dtype]
    assert layernorm.layernorm_queue_plan(M, N, code)[0] and not layernorm.layernorm_queue_plan(M - 1, N, code)[0]
    tdt = torch.float16 if dtype == inputs.FP16 else torch.bfloat16
    gen = torch.Generator(device=gpu_device).manual_seed(43)
    x = (0.5 + 2.0 * torch.randn((M, N), generator=gen, device=gpu_device)).to(tdt)
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(tdt)
    b = (0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(tdt)
    resident = layernorm.layernorm_fwd_tuned(x, w, b, EPS, threads) if threads else layernorm.layernorm_fwd_variant(x, w, b, EPS, Q)
    side = torch.cuda.Stream(device=gpu_device)
    torch.cuda.synchronize()
    y = torch.empty_like(x)
    for rep in range(3):
        H.say(f"layernorm queue auto {M}x{N} rep {rep}")
        y.fill_(3.0)
        layernorm.layernorm_fwd(x, w, b, EPS, y)
        assert torch.equal(y.view(torch.int16), resident.view(torch.int16))
        with torch.cuda.stream(side):
            side.wait_stream(torch.cuda.current_stream())
            ys = layernorm.layernorm_fwd(x, w, b, EPS)
        side.synchronize()
        assert torch.equal(ys.view(torch.int16), resident.view(torch.int16))
    rows = torch.tensor([0, 1, 7, 8, 15, 16, M // 2, M - 17, M - 1], device=gpu_device)
    as_u16 = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    case = dict(dtype=dtype, x=as_u16(x[rows]), w=as_u16(w), b=as_u16(b))
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], EPS, dtype, stats=True)
    compare.check_layernorm_parity(as_u16(y[rows]), want, _scale(case, mean, rstd), dtype, f"sampled rows of {M}x{N}")


def test_automatic_path_on_two_streams_at_once(gpu_device):
    """layernorm_fwd on two streams whose kernels may overlap: each stream has its own block of
    the library's counters, so neither launch sees the other's tickets."""
    M, N = 16384, 4096
    gen = torch.Generator(device=gpu_device).manual_seed(47)
    xs = [(torch.randn((M, N), generator=gen, device=gpu_device) + k).to(torch.float16) for k in range(2)]
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(torch.float16)
    b = (0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(torch.float16)
    assert layernorm.layernorm_queue_plan(M, N, layernorm.LAYERNORM_DTYPE_FP16)[0]
    resident = [layernorm.layernorm_fwd_tuned(x, w, b, EPS, 256) for x in xs]
    ys = [torch.empty_like(x) for x in xs]
    streams = [torch.cuda.Stream(device=gpu_device) for _ in xs]
    torch.cuda.synchronize()
    H.say("layernorm queue auto on two streams")
    for rep in range(6):
        for k, s in enumerate(streams):
            with torch.cuda.stream(s):
                layernorm.layernorm_fwd(xs[k], w, b, EPS, ys[k])
    torch.cuda.synchronize()
    for k in range(2):
        assert torch.equal(ys[k].view(torch.int16), resident[k].view(torch.int16))


def test_a_captured_call_does_not_use_the_shared_counters(gpu_device):
    """Under stream capture the automatic path takes the resident kernel (a graph may be replayed
    next to anything) and the forced variant reports that it cannot run; the replays give the bits
    of the eager call."""
    M, N = 16384, 4096
    gen = torch.Generator(device=gpu_device).manual_seed(53)
    x = torch.randn((M, N), generator=gen, device=gpu_device).to(torch.float16)
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(torch.float16)
    b = (0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(torch.float16)
    y = torch.empty_like(x)
    layernorm.layernorm_fwd(x, w, b, EPS, y)
    torch.cuda.synchronize()
    H.say("layernorm queue under capture")
    graph = torch.cuda.CUDAGraph()
    refused = []
    with torch.cuda.graph(graph):
        layernorm.layernorm_fwd(x, w, b, EPS, y)
        try:
            layernorm.layernorm_fwd_variant(x, w, b, EPS, Q, y)
        except layernorm.LayerNormError as e:
            refused.append(e.status)
    torch.cuda.synchronize()
    assert refused == [layernorm.LAYERNORM_ERR_UNSUPPORTED]
    for rep in range(3):
        x.copy_(torch.randn((M, N), generator=gen, device=gpu_device).to(torch.float16))
        y.fill_(3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = layernorm.layernorm_fwd(x, w, b, EPS)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
