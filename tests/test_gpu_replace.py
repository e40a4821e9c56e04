"""GPU parity of dgc_decompress_replace_regions: the dense aggregate of every iteration is
written in place of the one before, in one launch, and must equal the oracle's fresh sum
(zeros, then every payload added in worker order) bit for bit, whatever the aggregate of
the iteration before looked like.  Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import Pair, say

pytestmark = pytest.mark.gpu

SORTED = B.DGC_FLAG_SORTED_OUTPUT


def _run(gs, N, densities, seed, flags=0, scales=None, layout_density=None, warm=False, workers_per_iteration=None,
         reverse_previous=False, reshape=None, **extra):
    """One Pair per worker and per parity of the iteration (so that the previous payloads stay
    intact); every iteration replaces the aggregate and is compared with the oracle."""
    import torch
    lay_d = layout_density if layout_density is not None else max(densities) * 4
    kw = dict(momentum=0.9, density=densities[0], seed=seed, num_workers=N, flags=flags, **extra)
    shared = [S.gradient(gs, seed, 999, it, scales) for it in range(len(densities))]
    # two payload buffers per worker: iteration it writes into set it % 2
    workers = [[Pair(gs.offsets, layout_density=lay_d, warmup_workspace=warm, **kw) for _ in range(2)]
               for _ in range(N)]
    for w in range(N):                                         # one state (u, v) per worker, shared by its two Pairs
        workers[w][1].u, workers[w][1].v = workers[w][0].u, workers[w][0].v
        workers[w][1].ou, workers[w][1].ov = workers[w][0].ou, workers[w][0].ov
    acc = B.Dgc(B.make_config(**{k: v for k, v in kw.items()}), gs.offsets)
    acc.set_layout(workers[0][0].layout)
    dense = torch.zeros(gs.numel, device="cuda")
    previous = []
    for it, d in enumerate(densities):
        active = N if workers_per_iteration is None else workers_per_iteration[it]
        payloads, current = [], []
        for w in range(active):
            p = workers[w][it % 2]
            p.set_density(d)
            g = S.correlated_gradient(gs, seed, w, it, shared[it], scales=scales)
            if reshape is not None:
                reshape(g)
            res = p.step(g, it, check_state=False, label=f"replace it{it} w{w}")
            assert not res.overflow
            payloads.append(O.flatten_payload(res))
            current.append(p)
        acc.dgc_set_density(d)
        before = previous[::-1] if reverse_previous else previous       # the order of the previous payloads is free
        acc.dgc_decompress_replace_regions(dense, [p.out_idx for p in current], [p.out_val for p in current],
                                           [p.out_counts for p in current], [p.out_idx for p in before],
                                           [p.out_counts for p in before])
        expect = np.zeros(gs.numel, np.float32)
        O.decompress_accumulate(expect, payloads)
        got = dense.cpu().numpy()
        bad = np.flatnonzero(got.view(np.uint32) != expect.view(np.uint32))
        assert bad.size == 0, (it, d, bad[:5], got[bad[:5]], expect[bad[:5]])
        say(f"[replace] iteration {it} density {d}: {sum(i.size for i, _ in payloads)} pairs of {active} workers")
        previous = current
    acc.close()
    for pw in workers:
        for p in pw:
            p.close()


@pytest.mark.parametrize("flags", [0, SORTED])
@pytest.mark.parametrize("N,densities", [(1, [0.001, 0.001, 0.001]), (4, [0.002, 0.002, 0.002]),
                                         (16, [0.001, 0.001]), (3, [0.0625, 0.0625, 0.0625]),
                                         (6, [0.25, 0.0625, 0.002, 0.001, 0.25]),
                                         # 0.4 % of eight workers: more pairs per range than the 512-thread form holds
                                         (8, [0.004, 0.004, 0.001]),
                                         # 0.4 % of sixteen: more than any form holds, whole ranges are rewritten,
                                         # also in the first call at 0.1 %, whose previous payloads are long
                                         (16, [0.004, 0.004, 0.001, 0.001])])
def test_replace_equals_a_fresh_sum(N, densities, flags):
    gs = S.ragged_set(41, tensors=12, max_numel=400000)
    _run(gs, N, densities, 200 + N, flags=flags, layout_density=max(0.04, max(densities)), sample_min=1024,
         sample_max=8192)


def test_replace_with_more_pairs_than_a_workgroup_holds():
    """Eight payloads at 0.4 % whose large elements all sit at the front of their tensors: the first
    range of a tensor gets several times the pairs the density lets expect, more than registers and
    accumulator hold, and takes the general path (previous indices cleared first)."""
    gs = S.ragged_set(42, tensors=10, max_numel=400000)

    def front_heavy(g):
        for a, b in zip(gs.offsets[:-1], gs.offsets[1:]):
            g[a:a + min(60000, (b - a) // 4)] *= np.float32(1000.0)

    _run(gs, 8, [0.004, 0.004, 0.004], 77, layout_density=0.04, sample_min=1024, sample_max=8192, reshape=front_heavy)


def test_replace_with_the_previous_payloads_in_another_order():
    gs = S.ragged_set(44, tensors=12, max_numel=300000)
    _run(gs, 5, [0.002, 0.002, 0.002], 93, reverse_previous=True, layout_density=0.02, sample_min=1024,
         sample_max=8192)


def test_replace_with_a_changing_number_of_workers():
    gs = S.ragged_set(43, tensors=14, max_numel=300000)
    _run(gs, 8, [0.002, 0.002, 0.002, 0.002], 91, workers_per_iteration=[8, 2, 5, 1], layout_density=0.02,
         sample_min=1024, sample_max=8192)


def test_replace_resnet50_shape_sixteen_workers():
    gs = S.resnet50_set()
    _run(gs, 16, [0.001, 0.001, 0.001], 62, scales=S.tensor_scales(gs, 62), layout_density=0.001)
