"""Seeded random scenarios of the receive side against the oracle: a handful of workers with
random tensor sizes, densities on both sides of the 0.5 % switch between the two merge
kernels, sorted and unsorted payloads, with and without the staging workspace; over a few
iterations the dense vector is accumulated into, cleared, replaced, or a parameter vector
is stepped, in random order, and must hold the oracle's bits after every call.
Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from tests.parity import Pair

pytestmark = pytest.mark.gpu

DENSITIES = [0.001, 0.004, 0.006, 0.02, 0.1, 0.5]


@pytest.mark.parametrize("seed", range(24))
def test_random_receive_scenario(seed):
    import torch
    rng = np.random.default_rng([seed, 777])
    T = int(rng.integers(1, 10))
    sizes = [int(np.exp(rng.uniform(0.0, np.log(150000.0)))) for _ in range(T)]
    if rng.random() < 0.5:
        sizes.append(int(rng.integers(40000, 300000)))             # several emit parts in one tensor
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    n = int(offsets[-1])
    N = int(rng.integers(1, 13))
    flags = B.DGC_FLAG_SORTED_OUTPUT if rng.random() < 0.4 else 0
    warm = bool(rng.random() < 0.5)
    kw = dict(momentum=0.9, density=0.001, seed=int(rng.integers(0, 2 ** 31)), num_workers=N, flags=flags,
              sample_min=256, sample_max=4096)
    # two payload buffers per worker (the previous iteration's lists stay intact), one state
    workers = [[Pair(offsets, layout_density=1.0, warmup_workspace=warm, **kw) for _ in range(2)] for _ in range(N)]
    for pw in workers:
        pw[1].u, pw[1].v, pw[1].ou, pw[1].ov = pw[0].u, pw[0].v, pw[0].ou, pw[0].ov
    acc = B.Dgc(B.make_config(**kw), offsets)
    acc.set_layout(workers[0][0].layout)
    dense = torch.zeros(n, device="cuda")
    expect = np.zeros(n, np.float32)
    theta0 = rng.standard_normal(n).astype(np.float32)
    theta = torch.from_numpy(theta0).cuda()
    theta_expect = theta0.copy()
    # `previous`: the payloads (Pairs) outside whose indices `dense` is zero; their buffers are slot `held`
    previous, held = [], 0
    shared = rng.standard_normal(n).astype(np.float32)
    for it in range(5):
        d = float(rng.choice(DENSITIES))
        active = int(rng.integers(1, N + 1))
        slot = 1 - held                                            # never the buffers `previous` lives in
        current, payloads = [], []
        for w in range(active):
            p = workers[w][slot]
            p.set_density(d)
            g = (0.5 * shared + rng.standard_t(3, n)).astype(np.float32)
            res = p.step(g, it, check_state=False, label=f"receive seed={seed} it{it} w{w} d={d}")
            assert not res.overflow
            payloads.append(O.flatten_payload(res))
            current.append(p)
        lists = ([p.out_idx for p in current], [p.out_val for p in current], [p.out_counts for p in current])
        acc.dgc_set_density(d)
        op = str(rng.choice(["replace", "accumulate", "clear_then_accumulate", "sgd"]))
        reset = False
        if op == "replace":
            acc.dgc_decompress_replace_regions(dense, *lists, [p.out_idx for p in previous],
                                               [p.out_counts for p in previous])
            expect[:] = 0.0
            O.decompress_accumulate(expect, payloads)
            previous, held = current, slot
        elif op == "sgd":
            lr = float(rng.choice([0.01, 0.5]))
            acc.dgc_sparse_sgd_apply_regions(theta, lr, *lists)
            O.sparse_sgd_apply(theta_expect, payloads, lr)
        else:
            if op == "clear_then_accumulate" and previous:
                acc.dgc_dense_clear_regions(dense, [p.out_idx for p in previous], [p.out_counts for p in previous])
                expect[:] = 0.0
                previous = []
            reset = bool(previous)                                 # on top of an aggregate: two calls' payloads
            acc.dgc_decompress_accumulate_regions(dense, *lists)
            O.decompress_accumulate(expect, payloads)
            previous, held = current, slot
        got = dense.cpu().numpy()
        bad = np.flatnonzero(got.view(np.uint32) != expect.view(np.uint32))
        assert bad.size == 0, (seed, it, op, d, active, bad[:5], got[bad[:5]], expect[bad[:5]])
        assert np.array_equal(theta.cpu().numpy().view(np.uint32), theta_expect.view(np.uint32)), (seed, it, op)
        if reset:                                                  # start over from a zero aggregate
            dense.zero_()
            expect[:] = 0.0
            previous = []
    acc.close()
    for pw in workers:
        for p in pw:
            p.close()
