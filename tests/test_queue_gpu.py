"""The work-queue kernel (RMSNORM_VARIANT_QUEUE): resident workgroups that draw rows from
counters in device memory.  Checked here: parity with the oracle on every chunk count it is
built for, launch shapes that stress the row bookkeeping (more workgroups than rows, blocks
longer than the batch, one shard, 32 shards, a last block that is short), that the counters are
back at zero after every launch, that the bits equal those of one workgroup per row (the
arithmetic is the same, only the assignment of rows differs), two launches on two streams with
a workspace each, the automatic path at a size where it takes this kernel, and that a call
under graph capture takes another kernel."""
import numpy as np
import pytest
import torch

import gpu_harness as H
import oracle
import compare
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu

EPS = 1e-5


def _run_workspace(xd, wd, ws, plan=None, y=None):
    if plan is None:
        return binding.rmsnorm_fwd_workspace(xd, wd, EPS, ws, y)
    grid, shards, block_rows, prefetch = plan
    return binding.rmsnorm_fwd_queue_tuned(xd, wd, EPS, ws, grid, shards, block_rows, prefetch, y)


def _check(case, device, plans):
    dtype = case["dtype"]
    M, N = case["M"], case["N"]
    want = oracle.rmsnorm_oracle(case["x"], case["w"], EPS, dtype, 0)
    xd = H.to_device(case["x"], dtype, device)
    wd = H.to_device(case["w"], dtype, device)
    ws = binding.new_workspace(device)
    flat = H.to_host(binding.rmsnorm_fwd_tuned(xd, wd, EPS, 512), dtype)
    for plan in plans:
        H.say(f"queue {case['name']} plan={plan}")
        whole, y = H.alloc_guarded(M, N, dtype, device)
        _run_workspace(xd, wd, ws, plan, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype), f"{case['name']} {plan}: wrote outside y"
        got = H.to_host(y, dtype)
        compare.check_parity(got, want, dtype, f"{case['name']} {plan}")
        assert np.array_equal(got, flat), f"{case['name']} {plan}: bits differ from one workgroup per row"
        assert int(ws.abs().max().item()) == 0, f"{case['name']} {plan}: counters not back at zero"


# chunks per thread 2 .. 8 (rows of 513 .. 4096 vectors), exact and ragged last chunks
SHAPES = [
    (inputs.BF16, 700, 8192),     # 1024 vectors: 2 full chunks (the headline row)
    (inputs.BF16, 301, 5120),     # 640 vectors: 2 chunks, the second ragged
    (inputs.FP16, 129, 12288),    # 1536 vectors: 3 chunks
    (inputs.FP16, 77, 13824),     # 1728 vectors: 4 chunks, ragged
    (inputs.BF16, 65, 20480),     # 2560 vectors: 5 chunks
    (inputs.FP32, 97, 11264),     # 2816 vectors: 6 chunks, ragged
    (inputs.FP16, 40, 28672),     # 3584 vectors: 7 chunks
    (inputs.BF16, 50, 32768),     # 4096 vectors: 8 chunks
    (inputs.FP32, 257, 4096),     # 1024 vectors in fp32
    (inputs.FP32, 33, 16384),     # 4096 vectors in fp32
    (inputs.FP16, 520, 4104),     # 513 vectors: the shortest row the kernel takes
]


@pytest.mark.parametrize("dtype,M,N", SHAPES)
def test_parity_on_every_chunk_count(gpu_device, dtype, M, N):
    case = inputs.random_case(6, 900 + N % 97, M, N, dtype, EPS)
    _check(case, gpu_device, [None, (64, 16, 8, False), (48, 8, 4, True)])


@pytest.mark.parametrize("M", [1, 2, 7, 63, 64, 65, 1000, 1025, 2049])
def test_row_bookkeeping(gpu_device, M):
    """Batches around every boundary of the bookkeeping, under launch shapes with one member per
    shard, more workgroups than rows, blocks longer than the batch, one shard and 32 shards."""
    case = inputs.random_case(6, 950, M, 8192, inputs.BF16, EPS)
    plans = [(16, 16, 8, False), (512, 16, 8, False), (512, 16, 8, True), (96, 32, 1, False),
             (7, 1, 2, True), (3, 3, 1024, False), (64, 32, 64, True), (30, 5, 16, False)]
    _check(case, gpu_device, plans)


def test_invalid_plans_and_workspaces(gpu_device):
    case = inputs.random_case(6, 960, 8, 8192, inputs.BF16, EPS)
    xd = H.to_device(case["x"], inputs.BF16, gpu_device)
    wd = H.to_device(case["w"], inputs.BF16, gpu_device)
    ws = binding.new_workspace(gpu_device)
    for plan in [(10, 16, 8, False), (48, 32, 8, False), (64, 0, 8, False), (64, 33, 8, False),
                 (64, 16, 3, False), (64, 16, 0, False), (0, 1, 1, False), (1 << 17, 1, 1, False)]:
        with pytest.raises(binding.RmsnormError) as e:
            _run_workspace(xd, wd, ws, plan)
        assert e.value.status == binding.RMSNORM_ERR_INVALID_ARG, plan
    small = torch.zeros(100, dtype=torch.int32, device=gpu_device)
    with pytest.raises(binding.RmsnormError) as e:
        binding.rmsnorm_fwd_workspace(xd, wd, EPS, small)
    assert e.value.status == binding.RMSNORM_ERR_INVALID_ARG
    odd = torch.zeros(8192, dtype=torch.uint8, device=gpu_device)[1:4097 + 1]
    with pytest.raises(binding.RmsnormError) as e:
        binding.rmsnorm_fwd_workspace(xd, wd, EPS, odd)
    assert e.value.status == binding.RMSNORM_ERR_INVALID_ARG
    # rows the kernel does not take: too short, too long, not 16-byte aligned
    for N in (4096, 32776, 8191):
        c = inputs.random_case(6, 961, 4, N, inputs.BF16, EPS)
        with pytest.raises(binding.RmsnormError) as e:
            binding.rmsnorm_fwd_workspace(H.to_device(c["x"], inputs.BF16, gpu_device),
                                          H.to_device(c["w"], inputs.BF16, gpu_device), EPS, ws)
        assert e.value.status == binding.RMSNORM_ERR_UNSUPPORTED, N
    torch.cuda.synchronize()
    assert int(ws.abs().max().item()) == 0


def test_in_place_and_repeated_runs_are_bit_identical(gpu_device):
    case = inputs.random_case(6, 970, 3000, 8192, inputs.FP16, EPS)
    xd = H.to_device(case["x"], inputs.FP16, gpu_device)
    wd = H.to_device(case["w"], inputs.FP16, gpu_device)
    ws = binding.new_workspace(gpu_device)
    first = H.to_host(binding.rmsnorm_fwd_workspace(xd, wd, EPS, ws), inputs.FP16)
    for k in range(3):
        H.say(f"queue repeat {k}")
        again = H.to_host(binding.rmsnorm_fwd_workspace(xd, wd, EPS, ws), inputs.FP16)
        assert np.array_equal(again, first)
    H.say("queue in place")
    binding.rmsnorm_fwd_workspace(xd, wd, EPS, ws, xd)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(xd, inputs.FP16), first)


def test_two_streams_with_a_workspace_each(gpu_device):
    cases = [inputs.random_case(6, 980 + k, 4096, 8192, inputs.BF16, EPS) for k in range(2)]
    xs = [H.to_device(c["x"], inputs.BF16, gpu_device) for c in cases]
    ws_ = [H.to_device(c["w"], inputs.BF16, gpu_device) for c in cases]
    ys = [torch.empty_like(x) for x in xs]
    spaces = [binding.new_workspace(gpu_device) for _ in cases]
    flat = [H.to_host(binding.rmsnorm_fwd_tuned(x, w, EPS, 512), inputs.BF16) for x, w in zip(xs, ws_)]
    streams = [torch.cuda.Stream(device=gpu_device) for _ in cases]
    torch.cuda.synchronize()
    H.say("queue on two streams")
    for rep in range(4):
        for k, s in enumerate(streams):
            with torch.cuda.stream(s):
                binding.rmsnorm_fwd_workspace(xs[k], ws_[k], EPS, spaces[k], ys[k])
    torch.cuda.synchronize()
    for k in range(2):
        assert np.array_equal(H.to_host(ys[k], inputs.BF16), flat[k])
        assert int(spaces[k].abs().max().item()) == 0


def test_automatic_path_on_two_streams_at_once(gpu_device):
    """rmsnorm_fwd on two streams whose kernels may overlap: each stream gets its own block of
    the library's counters, so neither launch sees the other's tickets."""
    cases = [inputs.random_case(6, 985 + k, 6144, 8192, inputs.BF16, EPS) for k in range(2)]
    xs = [H.to_device(c["x"], inputs.BF16, gpu_device) for c in cases]
    ws_ = [H.to_device(c["w"], inputs.BF16, gpu_device) for c in cases]
    ys = [torch.empty_like(x) for x in xs]
    flat = [H.to_host(binding.rmsnorm_fwd_tuned(x, w, EPS, 512), inputs.BF16) for x, w in zip(xs, ws_)]
    streams = [torch.cuda.Stream(device=gpu_device) for _ in cases]
    torch.cuda.synchronize()
    H.say("queue auto on two streams")
    for rep in range(6):
        for k, s in enumerate(streams):
            with torch.cuda.stream(s):
                assert binding.rmsnorm_select_variant(xs[k], ws_[k], ys[k]) == binding.RMSNORM_VARIANT_QUEUE
                binding.rmsnorm_fwd(xs[k], ws_[k], EPS, ys[k])
    torch.cuda.synchronize()
    for k in range(2):
        assert np.array_equal(H.to_host(ys[k], inputs.BF16), flat[k])


def test_automatic_path_takes_the_queue_for_large_launches(gpu_device):
    """96 MiB of 16 KiB rows: rmsnorm_fwd runs the work-queue kernel on the stream's own counters
    (on the default stream, on a side stream, several times in a row), with the bits of one
    workgroup per row; the forced variant does the same."""
    M, N = 6144, 8192
    case = inputs.random_case(6, 990, M, N, inputs.BF16, EPS)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], EPS, inputs.BF16, 0)
    xd = H.to_device(case["x"], inputs.BF16, gpu_device)
    wd = H.to_device(case["w"], inputs.BF16, gpu_device)
    takes, grid, shards, block_rows, prefetch = binding.rmsnorm_queue_plan(M, N, binding.RMSNORM_DTYPE_BF16)
    assert takes and grid % shards == 0
    assert binding.rmsnorm_select_variant(xd, wd, torch.empty_like(xd)) == binding.RMSNORM_VARIANT_QUEUE
    flat = H.to_host(binding.rmsnorm_fwd_tuned(xd, wd, EPS, 512), inputs.BF16)
    compare.check_parity(flat, want, inputs.BF16, "one workgroup per row")
    side = torch.cuda.Stream(device=gpu_device)
    for rep in range(3):
        H.say(f"queue auto rep {rep}")
        got = H.to_host(binding.rmsnorm_fwd(xd, wd, EPS), inputs.BF16)
        assert np.array_equal(got, flat)
        forced = H.to_host(binding.rmsnorm_fwd_variant(xd, wd, EPS, binding.RMSNORM_VARIANT_QUEUE), inputs.BF16)
        assert np.array_equal(forced, flat)
        with torch.cuda.stream(side):
            y = binding.rmsnorm_fwd(xd, wd, EPS)
        side.synchronize()
        assert np.array_equal(H.to_host(y, inputs.BF16), flat)


def test_automatic_path_takes_the_queue_for_rows_under_16_kib_from_320_mib_on(gpu_device):
    """32768 rows of 10 KiB (320 MiB of x): the automatic path runs the work-queue kernel, with
    the bits of 512 threads per row; one row less and it does not.  A sample of rows against
    the oracle."""
    M, N = 32768, 5120
    bf16 = binding.RMSNORM_DTYPE_BF16
    assert binding.rmsnorm_queue_plan(M, N, bf16)[0] and not binding.rmsnorm_queue_plan(M - 1, N, bf16)[0]
    gen = torch.Generator(device=gpu_device).manual_seed(41)
    x = torch.randn((M, N), generator=gen, device=gpu_device).to(torch.bfloat16)
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(torch.bfloat16)
    assert binding.rmsnorm_select_variant(x, w, torch.empty_like(x)) == binding.RMSNORM_VARIANT_QUEUE
    H.say("queue auto, 10 KiB rows")
    got = binding.rmsnorm_fwd(x, w, EPS)
    flat = binding.rmsnorm_fwd_tuned(x, w, EPS, 512)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), flat.view(torch.int16))
    rows = torch.tensor([0, 1, 7, 8, 4095, 4096, 20000, M - 9, M - 1], device=gpu_device)
    xs = x[rows].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    ws = w.view(torch.int16).cpu().numpy().view(np.uint16)
    want = oracle.rmsnorm_oracle(xs, ws, EPS, inputs.BF16, 0)
    compare.check_parity(got[rows].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), want, inputs.BF16,
                         "sampled rows of 32768 x 5120")


def test_a_captured_call_does_not_use_the_shared_counters(gpu_device):
    """Under stream capture the automatic path takes the one-workgroup-per-row kernel (a graph
    may be replayed next to anything) and the forced variant reports that it cannot run; the
    replays give the bits of the eager call."""
    M, N = 6144, 8192
    gen = torch.Generator(device=gpu_device).manual_seed(99)
    x = torch.randn((M, N), generator=gen, device=gpu_device).to(torch.bfloat16)
    w = (1.0 + 0.1 * torch.randn(N, generator=gen, device=gpu_device)).to(torch.bfloat16)
    y = torch.empty_like(x)
    binding.rmsnorm_fwd(x, w, EPS, y)
    torch.cuda.synchronize()
    H.say("queue under capture")
    graph = torch.cuda.CUDAGraph()
    refused = []
    with torch.cuda.graph(graph):
        binding.rmsnorm_fwd(x, w, EPS, y)
        try:
            binding.rmsnorm_fwd_variant(x, w, EPS, binding.RMSNORM_VARIANT_QUEUE, y)
        except binding.RmsnormError as e:
            refused.append(e.status)
    torch.cuda.synchronize()
    assert refused == [binding.RMSNORM_ERR_UNSUPPORTED]
    for rep in range(3):
        x.copy_(torch.randn((M, N), generator=gen, device=gpu_device).to(torch.bfloat16))
        y.fill_(3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = binding.rmsnorm_fwd(x, w, EPS)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
