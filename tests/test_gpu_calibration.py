"""The calibration streams move what they say they move: the copy reproduces its source byte for byte (its tiles are
handed to the XCDs in runs, a permutation of the workgroups: sizes below one group of runs, at exact multiples of it
and with a partial last group), the write fills exactly `bytes`, the read touches nothing."""
import pytest
import torch

import paper_2110_05722_amd as L
from tests._util import dev, say

pytestmark = pytest.mark.gpu

TILE = 1024                       # bytes per workgroup
GROUP = 8 * 1024 * TILE           # bytes per group of eight runs of 1024 tiles


@pytest.mark.parametrize("nbytes", [16, TILE, 3 * TILE + 48, GROUP, 2 * GROUP, 2 * GROUP + 5 * TILE + 16])
def test_copy_write_read(nbytes):
    say(f"[calibration] streams over {nbytes} bytes")
    d = dev()
    g = torch.Generator(device="cpu").manual_seed(nbytes % 1000)
    src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, generator=g).to(d)
    dst = torch.full((nbytes + 64,), 7, dtype=torch.uint8, device=d)
    L.lsq_calib_stream("copy", dst, src, nbytes)
    assert torch.equal(dst[:nbytes], src[:nbytes])
    assert bool((dst[nbytes:] == 7).all()), "the copy wrote past its length"
    dst.fill_(7)
    L.lsq_calib_stream("write", dst, None, nbytes)
    assert bool((dst[:nbytes].view(torch.int16) == 0x3C00).all())
    assert bool((dst[nbytes:] == 7).all()), "the write went past its length"
    sink = torch.zeros(1, dtype=torch.int32, device=d)
    before = src.clone()
    L.lsq_calib_stream("read", sink, src, nbytes)
    assert int(sink.item()) == 0 and torch.equal(src, before)
    L.lsq_calib_stream("empty", sink, None, 0)
    torch.cuda.synchronize()
