"""Seeded random configurations of the whole path against the oracle: tensor sizes from
one element to a few tiles, every flag combination, densities from 0.1 % to 100 %,
sample blocks from 1 to 64, clipping on and off, payload capacities that overflow.
Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from tests.parity import Pair, check_overflow_invariants

pytestmark = pytest.mark.gpu


def random_case(seed: int):
    rng = np.random.default_rng([seed, 4242])
    T = int(rng.integers(1, 12))
    sizes = [int(np.exp(rng.uniform(0.0, np.log(40000.0)))) for _ in range(T)]
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    flags = 0
    for f in (B.DGC_FLAG_NESTEROV, B.DGC_FLAG_NO_FACTOR_MASKING, B.DGC_FLAG_EXACT_SELECT, B.DGC_FLAG_SORTED_OUTPUT):
        if rng.random() < 0.4:
            flags |= f
    block = int(rng.choice([1, 2, 8, 32, 64]))
    smin = int(rng.choice([64, 256, 4096]))
    kw = dict(momentum=float(rng.choice([0.0, 0.5, 0.9])), density=float(rng.choice([0.001, 0.01, 0.1, 0.5, 1.0])),
              seed=int(rng.integers(0, 2 ** 40)), flags=flags, sample_block=block, sample_min=max(smin, block),
              sample_max=max(smin, block) * int(rng.choice([1, 4])), sample_ratio=float(rng.choice([0.01, 0.1])))
    if rng.random() < 0.4:
        kw.update(clip_threshold=float(rng.choice([0.01, 1.0, 100.0])), num_workers=int(rng.integers(1, 9)))
    if rng.random() < 0.3:
        kw.update(refine_alpha=float(rng.choice([1.0, 1.5, 3.0])))
    tight = rng.random() < 0.25                           # capacities below what will pass
    return rng, offsets, sizes, kw, tight


@pytest.mark.parametrize("warm", [False, True])      # True: workspace with the staging arrays of the warm-up densities
@pytest.mark.parametrize("seed", range(48))
def test_random_configuration(seed, warm):
    rng, offsets, sizes, kw, tight = random_case(seed)
    n = int(offsets[-1])
    if tight:
        caps = [max(1, O.topk_count(kw["density"], s) // 2) for s in sizes]
        p = Pair(offsets, capacities=caps, warmup_workspace=warm, **kw)
    else:
        p = Pair(offsets, layout_density=1.0, warmup_workspace=warm, **kw)       # room for anything a small sample lets through
    scale = float(rng.choice([1e-3, 1.0, 30.0]))
    wander = (not tight) and rng.random() < 0.5            # another density every iteration, one state
    for it in range(3):
        if wander and it:
            p.set_density(float(rng.choice([0.001, 0.004, 0.006, 0.01, 0.1, 0.5, 1.0])))
        g = (scale * rng.standard_t(3, n)).astype(np.float32)
        if rng.random() < 0.3:
            g[rng.random(n) < 0.7] = 0.0                  # mostly zero: thresholds of 0, empty regions
        u0 = p.u.cpu().numpy().copy()
        v0 = p.v.cpu().numpy().copy()
        res = p.step(g, it + int(rng.integers(0, 1000)) * (it == 2), label=f"random seed={seed} it{it} {kw}")
        if res.overflow and not p.sorted:
            check_overflow_invariants(p, g, u0, v0)
            break                                         # the two sides' states differ from here on (order-dependent)
    p.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_large_configuration(seed):
    """Millions of elements in a few dozen tensors of very different sizes: thousands of wave
    tiles per tensor, hundreds of emit parts, regions of 10^5 pairs; compress over three
    iterations with the density changing, then the receive side of three workers."""
    import torch
    rng = np.random.default_rng([seed, 90210])
    T = int(rng.integers(2, 40))
    sizes = [int(np.exp(rng.uniform(np.log(10.0), np.log(3.0e6)))) for _ in range(T)]
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    n = int(offsets[-1])
    flags = 0
    for f in (B.DGC_FLAG_NESTEROV, B.DGC_FLAG_NO_FACTOR_MASKING, B.DGC_FLAG_SORTED_OUTPUT):
        if rng.random() < 0.3:
            flags |= f
    warm = bool(rng.random() < 0.6)
    kw = dict(momentum=0.9, density=0.001, seed=int(rng.integers(0, 2 ** 40)), flags=flags, num_workers=3)
    if rng.random() < 0.4:
        kw.update(clip_threshold=float(rng.choice([0.5, 50.0])))
    if seed % 2:                                          # the re-threshold on records and mask words side by side
        kw.update(refine_alpha=float(1.0 + seed % 3))
    workers = [Pair(offsets, layout_density=0.25, warmup_workspace=warm, **kw) for _ in range(3)]
    shared = rng.standard_t(3, n).astype(np.float32)
    densities = [float(rng.choice([0.001, 0.004, 0.02, 0.1])) for _ in range(3)]
    payloads = []
    for it, d in enumerate(densities):
        payloads = []
        for w, p in enumerate(workers):
            p.set_density(d)
            g = (0.01 * (0.5 * shared + rng.standard_t(3, n))).astype(np.float32)
            res = p.step(g, it, check_state=(w == 0), label=f"large seed={seed} it{it} w{w} d={d} n={n} T={T}")
            assert not res.overflow
            payloads.append(O.flatten_payload(res))
    acc = B.Dgc(B.make_config(**kw), offsets)
    acc.set_layout(workers[0].layout)
    acc.dgc_set_density(densities[-1])
    dense = torch.zeros(n, device="cuda")
    lists = ([p.out_idx for p in workers], [p.out_val for p in workers], [p.out_counts for p in workers])
    expect = np.zeros(n, np.float32)
    O.decompress_accumulate(expect, payloads)
    acc.dgc_decompress_replace_regions(dense, *lists)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32)), "replace"
    acc.dgc_dense_clear_regions(dense, lists[0], lists[2])
    assert not dense.any().item(), "clear"
    acc.dgc_decompress_accumulate_regions(dense, *lists)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32)), "accumulate"
    acc.close()
    for p in workers:
        p.close()
