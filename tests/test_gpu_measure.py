"""The two measurement kernels behind bench.py's `ceilings` block: the copy really copies
(read once, written `fanout` times), the MFMA loop runs and reports its operation count."""
import pytest
import torch

import paper_2510_19470_amd as moe
from gpu_common import DEV, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fanout", [1, 2, 3])
def test_measure_copy_copies(fanout):
    n = (1 << 20) + 4096 + 16          # not a multiple of the 4 KB a block moves
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros(fanout * n + 64, dtype=torch.uint8, device=DEV)
    moe.moe_measure_copy(src, dst[:fanout * n], fanout)
    torch.cuda.synchronize()
    for c in range(fanout):
        assert torch.equal(dst[c * n:(c + 1) * n], src), c
    assert int(dst[fanout * n:].sum()) == 0                      # nothing past the copies
    say(f"  copy fanout {fanout}: {n} bytes, exact")


def test_measure_mfma_runs():
    blocks, iters = 16, 64
    sink = torch.full((blocks * 512,), 7.0, dtype=torch.float32, device=DEV)
    fl = moe.moe_measure_mfma(sink, blocks, iters, False)
    torch.cuda.synchronize()
    assert fl == blocks * 8 * iters * 32 * 2 * 32 * 32 * 16
    assert float(sink.abs().max()) == 0.0                        # zero operands: zero sums
    moe.moe_measure_mfma(sink, blocks, iters, True)
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all() and float(sink.abs().max()) > 0.0
