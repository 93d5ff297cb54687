"""Rows that are not 16-byte aligned, with enough of them for the resident ("walking") form of
the element-addressed kernels: every workgroup takes rows that start at one offset from a
128-byte line, lays its 16-byte slots out from that line and keeps its slices of the weight
(and bias) in registers.  Every thread count and number of slots per thread of that form, all
the offsets a row can have (odd N walks through them from row to row), bases off a boundary,
in place, and a row count that does not divide evenly; RMSNorm, softmax (whose kernel makes
the same cut per row, without residency) and LayerNorm against the CPU oracle, element by
element, in fp16, bf16 and fp32; also with y at another offset from a line than x (the cut
follows x, the stores straddle the lines)."""
import pytest
import torch

import compare
import gpu_harness as H
import oracle
import test_layernorm_gpu as LN
from paper_2603_21331_amd import binding, inputs, layernorm, softmax

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP16, inputs.BF16]
# N: 64 threads with 2, 3, 4 slots each; 256 with 2, 4, 6, 8; 512 with 5, 8; 1024 with 5, 7
# (RMSNorm) and 256 with 1..4, 512 with 3, 4, 1024 with 3, 4 (LayerNorm).
LENGTHS = [1025, 1537, 2047, 2057, 4097, 8191, 12289, 16383, 20481, 32767, 40961, 57343]
# the same slot counts in fp32
LENGTHS_FP32 = [513, 769, 1023, 1029, 2049, 4095, 6145, 8191, 10241, 16383, 20481, 28671]
CASES = [(N, d) for d in DTYPES for N in LENGTHS] + [(N, inputs.FP32) for N in LENGTHS_FP32]


def rows_for(N: int, dtype: int = inputs.FP16) -> int:
    """Enough rows for four per workgroup of the smallest grid LayerNorm's form takes (the
    larger of the two), and 37 more so that the last round is ragged."""
    want = 48 * 1024 / (inputs.DTYPE_BYTES[dtype] * N)
    per_cu = 1
    while per_cu < 0.55 * want:
        per_cu += 1
    return 4 * 256 * min(per_cu, 8) + 37


def layernorm_walks(N: int, dtype: int) -> bool:
    """More than 256 and at most 4096 whole 16-byte pieces per row."""
    return 256 < N * inputs.DTYPE_BYTES[dtype] // 16 <= 4096


@pytest.mark.parametrize("N,dtype", CASES)
def test_walking_form_matches_the_oracle(gpu_device, N, dtype):
    M = rows_for(N, dtype)
    case = inputs.layernorm_case(9, 1400 + 4 * dtype + N % 89, M, N, dtype, 1e-5, mean=0.5, std=1.5)
    xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
    wr, yr = H.alloc_guarded(M, N, dtype, gpu_device)
    ws, ys = H.alloc_guarded(M, N, dtype, gpu_device)
    wl, yl = H.alloc_guarded(M, N, dtype, gpu_device)
    walk_r = binding.rmsnorm_unaligned_walk_grid(xd, wd, yr)
    walk_l = layernorm.layernorm_unaligned_walk_grid(xd, wd, bd, yl)
    assert walk_r > 0 and walk_r % 64 == 0, "the RMSNorm call does not reach the walking form"
    assert (walk_l > 0 and walk_l % 64 == 0) == layernorm_walks(N, dtype)
    H.say(f"walking form {inputs.DTYPE_NAMES[dtype]} {M}x{N}: grids {walk_r}, {walk_l}")
    binding.rmsnorm_fwd(xd, wd, 1e-5, yr)
    softmax.softmax_fwd(xd, ys)
    layernorm.layernorm_fwd(xd, wd, bd, 1e-5, yl)
    torch.cuda.synchronize()
    for whole in (wr, ws, wl):
        assert H.guards_intact(whole, M, N, dtype), f"N={N}: wrote outside an output"
    compare.check_parity(H.to_host(yr, dtype), oracle.rmsnorm_oracle(case["x"], case["w"], 1e-5, dtype),
                         dtype, f"rmsnorm {M}x{N}")
    compare.check_softmax_parity(H.to_host(ys, dtype), oracle.softmax_oracle(case["x"], dtype), dtype,
                                 f"softmax {M}x{N}")
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    compare.check_layernorm_parity(H.to_host(yl, dtype), want, LN.scale_of(case, mean, rstd), dtype,
                                   f"layernorm {M}x{N}")


@pytest.mark.parametrize("dtype", DTYPES + [inputs.FP32])
@pytest.mark.parametrize("N,offset", [(4097, 3), (2050, 5), (8192, 1), (1026, 7), (2048, 40)])
def test_walking_form_off_a_boundary_in_place_and_without_bias(gpu_device, N, offset, dtype):
    """x and y `offset` elements past a 16-byte boundary (even N included: every row then
    starts at that one offset; 40 elements: whole 16-byte slots, but off the 128-byte lines),
    weight and bias at offsets of their own; then in place; then LayerNorm without a bias."""
    M = rows_for(N, dtype)
    td = H.torch_dtype(dtype)
    case = inputs.layernorm_case(9, 1460 + 4 * dtype + offset, M, N, dtype, 1e-5, mean=-0.25, std=2.0)
    xbuf = torch.zeros(M * N + 64, dtype=td, device=gpu_device)
    wbuf = torch.zeros(N + 16, dtype=td, device=gpu_device)
    bbuf = torch.zeros(N + 16, dtype=td, device=gpu_device)
    xd = xbuf[offset:offset + M * N].view(M, N)
    wd, bd = wbuf[1:1 + N], bbuf[2:2 + N]
    xd.copy_(H.to_device(case["x"], dtype, gpu_device))
    wd.copy_(H.to_device(case["w"], dtype, gpu_device))
    bd.copy_(H.to_device(case["b"], dtype, gpu_device))
    want_r = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-5, dtype)
    want_s = oracle.softmax_oracle(case["x"], dtype)
    want_l, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    want_n, _, _ = oracle.layernorm_oracle(case["x"], case["w"], None, 1e-5, dtype, stats=True)
    scale = LN.scale_of(case, mean, rstd)
    scale_n = LN.scale_of(dict(case, b=None), mean, rstd)

    wr, yr = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=offset)
    ws, ys = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=offset)
    wl, yl = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=offset)
    wn, yn = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=offset)
    assert binding.rmsnorm_unaligned_walk_grid(xd, wd, yr) > 0
    assert (layernorm.layernorm_unaligned_walk_grid(xd, wd, bd, yl) > 0) == layernorm_walks(N, dtype)
    H.say(f"walking form off a boundary {inputs.DTYPE_NAMES[dtype]} {M}x{N} offset {offset}")
    binding.rmsnorm_fwd_variant(xd, wd, 1e-5, binding.RMSNORM_VARIANT_UNALIGNED, yr)
    softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_UNALIGNED, ys)
    layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, layernorm.LAYERNORM_VARIANT_UNALIGNED, yl)
    layernorm.layernorm_fwd_variant(xd, wd, None, 1e-5, layernorm.LAYERNORM_VARIANT_UNALIGNED, yn)
    torch.cuda.synchronize()
    for whole in (wr, ws, wl, wn):
        assert H.guards_intact(whole, M, N, dtype, offset_elems=offset)
    compare.check_parity(H.to_host(yr, dtype), want_r, dtype, "rmsnorm off a boundary")
    compare.check_softmax_parity(H.to_host(ys, dtype), want_s, dtype, "softmax off a boundary")
    compare.check_layernorm_parity(H.to_host(yl, dtype), want_l, scale, dtype, "layernorm off a boundary")
    compare.check_layernorm_parity(H.to_host(yn, dtype), want_n, scale_n, dtype, "layernorm, no bias")

    # y one element further from the boundary than x: the rows are cut at x's lines and the
    # stores are element-aligned
    other = offset + 1
    wr, yr = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=other)
    ws, ys = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=other)
    wl, yl = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=other)
    assert binding.rmsnorm_unaligned_walk_grid(xd, wd, yr) > 0
    H.say(f"walking form, y at another offset {inputs.DTYPE_NAMES[dtype]} {M}x{N} offsets {offset}, {other}")
    binding.rmsnorm_fwd_variant(xd, wd, 1e-5, binding.RMSNORM_VARIANT_UNALIGNED, yr)
    softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_UNALIGNED, ys)
    layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, layernorm.LAYERNORM_VARIANT_UNALIGNED, yl)
    torch.cuda.synchronize()
    for whole in (wr, ws, wl):
        assert H.guards_intact(whole, M, N, dtype, offset_elems=other)
    compare.check_parity(H.to_host(yr, dtype), want_r, dtype, "rmsnorm, y at another offset")
    compare.check_softmax_parity(H.to_host(ys, dtype), want_s, dtype, "softmax, y at another offset")
    compare.check_layernorm_parity(H.to_host(yl, dtype), want_l, scale, dtype, "layernorm, y at another offset")

    for name, launch, check in (
            ("rmsnorm", lambda t: binding.rmsnorm_fwd_variant(t, wd, 1e-5, binding.RMSNORM_VARIANT_UNALIGNED, t),
             lambda got: compare.check_parity(got, want_r, dtype, "rmsnorm in place")),
            ("softmax", lambda t: softmax.softmax_fwd_variant(t, softmax.SOFTMAX_VARIANT_UNALIGNED, t),
             lambda got: compare.check_softmax_parity(got, want_s, dtype, "softmax in place")),
            ("layernorm", lambda t: layernorm.layernorm_fwd_variant(t, wd, bd, 1e-5,
                                                                    layernorm.LAYERNORM_VARIANT_UNALIGNED, t),
             lambda got: compare.check_layernorm_parity(got, want_l, scale, dtype, "layernorm in place"))):
        tbuf = xbuf.clone()
        t = tbuf[offset:offset + M * N].view(M, N)
        H.say(f"walking form in place: {name}")
        launch(t)
        torch.cuda.synchronize()
        assert torch.equal(tbuf[:offset], xbuf[:offset]) and torch.equal(tbuf[offset + M * N:], xbuf[offset + M * N:])
        check(H.to_host(t, dtype))
