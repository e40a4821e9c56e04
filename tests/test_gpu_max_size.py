"""The largest set a handle accepts (2^31 - 65536 elements, a little less here so that the last
tile is ragged: indices are int32 and every index computation of the kernels runs close to its
limit) through dgc_compress and the receive side, element by element against
the oracle.  One tensor of 2.1 G elements and two small ones behind it.  Needs about 40 GB of
device memory and 110 GB of host memory.  Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from tests.parity import Pair, say

pytestmark = pytest.mark.gpu

N_MAX = (1 << 31) - 65536


@pytest.mark.parametrize("density,iterations,warm", [(0.001, 2, False), (0.0625, 1, True)])
def test_largest_set_through_compress_and_receive_side(density, iterations, warm):
    """0.1 %: the slotted passes and the range kernel of the receive side; 6.25 %: the staged passes and the
    part kernels."""
    import torch
    n = N_MAX - 3
    offsets = [0, n - 70001, n - 1031, n]
    rng = np.random.default_rng(20171201)
    g = rng.standard_normal(n, dtype=np.float32)
    g[offsets[1]:] *= np.float32(0.01)                     # the small tensors on a scale of their own
    p = Pair(offsets, momentum=0.9, density=density, seed=9, num_workers=1, warmup_workspace=warm)
    for it in range(iterations):
        res = p.step(g, it, label=f"largest set it{it}")
        assert not res.overflow
        say(f"[max size] iteration {it}: {int(res.counts.sum())} pairs, last index {int(res.indices[2][-1])}")
    assert int(res.indices[0][-1]) > (1 << 31) - (1 << 22)  # the payload reaches the top of the index range
    del g
    expect = np.zeros(n, np.float32)
    O.decompress_accumulate(expect, [O.flatten_payload(res)])
    dense = torch.zeros(n, device="cuda")
    lists = ([p.out_idx], [p.out_val], [p.out_counts])
    p.dgc.dgc_decompress_accumulate_regions(dense, *lists)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    p.dgc.dgc_decompress_replace_regions(dense, *lists, [p.out_idx], [p.out_counts])
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    p.dgc.dgc_dense_clear_regions(dense, [p.out_idx], [p.out_counts])
    assert not bool(dense.any())
    p.close()
