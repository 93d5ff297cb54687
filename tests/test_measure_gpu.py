"""The measurement library's two copies on the GPU: every byte arrives, nothing beyond the last
byte is written, at sizes below one tile, of exactly one tile, with a ragged last tile and of
many tiles."""
import pytest
import torch

import gpu_harness as H
from paper_2603_21331_amd import measure

pytestmark = pytest.mark.gpu

SIZES = [16, 48, 8192 - 16, 8192, 8192 + 16, 3 * 8192 + 4080, (1 << 20) + 48, 64 << 20]


@pytest.mark.parametrize("nbytes", SIZES)
@pytest.mark.parametrize("entry", ["measure_copy", "measure_staged_copy"])
def test_copies_every_byte_and_nothing_more(gpu_device, entry, nbytes):
    H.say(f"{entry} {nbytes} bytes")
    gen = torch.Generator(device=gpu_device).manual_seed(nbytes % 1000)
    words = nbytes // 4
    src = torch.randint(-2**31, 2**31 - 1, (words,), generator=gen, device=gpu_device, dtype=torch.int32)
    guard = 64
    whole = torch.full((words + 2 * guard,), 0x5A5A5A5A, device=gpu_device, dtype=torch.int32)
    dst = whole[guard:guard + words]
    assert dst.data_ptr() % 16 == 0
    getattr(measure, entry)(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert bool((whole[:guard] == 0x5A5A5A5A).all()) and bool((whole[guard + words:] == 0x5A5A5A5A).all())
