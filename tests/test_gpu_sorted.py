"""GPU parity of the sorted payload (DGC_FLAG_SORTED_OUTPUT): every tensor's region
must hold the oracle's pairs in the oracle's order (ascending index), without any
sorting on the test's side, and a full region must keep the lowest indices.  Also the
receive side that merges payloads by element range, with and without the flag.
Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import Pair, say

pytestmark = pytest.mark.gpu

SORTED = B.DGC_FLAG_SORTED_OUTPUT


@pytest.mark.parametrize("flags", [SORTED, SORTED | B.DGC_FLAG_NESTEROV | B.DGC_FLAG_NO_FACTOR_MASKING,
                                   SORTED | B.DGC_FLAG_EXACT_SELECT])
@pytest.mark.parametrize("density", [0.001, 0.05, 1.0])
def test_sorted_ragged_set(flags, density):
    gs = S.ragged_set(3)
    p = Pair(gs.offsets, layout_density=max(density, 0.05), momentum=0.9, density=density, flags=flags,
             seed=11, sample_min=256, sample_max=2048, sample_block=16)
    for it in range(3):
        p.step(S.gradient(gs, 21, 0, it), it, label=f"sorted ragged flags={flags} d={density} it{it}")
    p.close()


def test_sorted_edge_sizes():
    for sizes in ([1], [1023], [1024], [1025], [4096, 3], [5, 1019, 1, 2047, 7], [32768, 32769, 1, 65536]):
        offsets = np.concatenate([[0], np.cumsum(sizes)])
        p = Pair(offsets, layout_density=1.0, momentum=0.9, density=0.3, seed=1, sample_min=64, sample_max=256,
                 flags=SORTED)
        rng = np.random.default_rng(sum(sizes))
        for it in range(2):
            p.step(rng.standard_normal(offsets[-1]).astype(np.float32), it, label=f"sorted sizes={sizes} it{it}")
        p.close()


def test_sorted_overflow_keeps_lowest_indices_like_the_oracle():
    gs = S.ragged_set(6, tensors=10)
    caps = [max(1, O.topk_count(0.05, s) // 2) for s in gs.sizes]
    p = Pair(gs.offsets, capacities=caps, momentum=0.9, density=0.05, seed=9,
             flags=SORTED | B.DGC_FLAG_EXACT_SELECT)
    u0 = (0.1 * S.gradient(gs, 23, 1, 0)).astype(np.float32)
    v0 = (0.1 * S.gradient(gs, 23, 2, 0)).astype(np.float32)
    p.set_state(u0, v0)
    for it in range(3):                                   # what overflowed stays in v and passes again
        res = p.step(S.gradient(gs, 23, 0, it), it, label=f"sorted overflow it{it}")
        assert res.overflow
    p.close()


def test_sorted_with_rethreshold():
    gs = S.ragged_set(12, tensors=14, max_numel=120000)
    p = Pair(gs.offsets, momentum=0.9, density=0.01, seed=21, sample_min=64, sample_max=64, sample_block=4,
             refine_alpha=1.0, flags=SORTED)
    refined = 0
    for it in range(4):
        res = p.step(S.gradient(gs, 26, 0, it), it, label=f"sorted refine it{it}")
        refined += sum(res.refined)
    assert refined >= 3
    p.close()


@pytest.mark.parametrize("flags", [SORTED, 0])
def test_payload_is_identical_on_every_run(flags):
    import torch
    gs = S.ragged_set(15, tensors=16, max_numel=300000)
    kw = dict(layout_density=0.02, momentum=0.9, density=0.01, seed=5, sample_min=256, sample_max=2048,
              flags=flags)
    g = [S.gradient(gs, 28, 0, it) for it in range(3)]
    runs = []
    for rep in range(3):
        p = Pair(gs.offsets, **kw)
        p.out_idx.fill_(-7)
        p.out_val.fill_(float("nan"))
        for it in range(3):
            p.dgc.dgc_compress(torch.from_numpy(g[it]).cuda(), p.u, p.v, p.out_idx, p.out_val, p.out_counts,
                               p.out_thr, it)
        runs.append((p.out_idx.cpu().numpy().copy(), p.out_val.cpu().numpy().view(np.uint32).copy(),
                     p.out_counts.cpu().numpy().copy()))
        p.close()
    for r in runs[1:]:
        for a, b in zip(runs[0], r):
            assert np.array_equal(a, b)


def test_sorted_resnet50_set_and_high_density_speech():
    gs = S.resnet50_set()
    scales = S.tensor_scales(gs, 31)
    p = Pair(gs.offsets, momentum=0.9, density=0.001, seed=31, flags=SORTED)
    for it in range(2):
        say(f"[sorted resnet50] iteration {it}")
        p.step(S.gradient(gs, 31, 0, it, scales), it, label=f"sorted resnet50 it{it}")
    p.close()
    gs = S.speech_set()
    scales = S.tensor_scales(gs, 51)
    p = Pair(gs.offsets, layout_density=0.25, momentum=0.9, density=0.25, seed=51, num_workers=8, flags=SORTED)
    for it in range(2):                                   # 25 % then 6.25 %: millions of pairs per tensor
        d = O.warmup_density(O.WARMUP_DENSITIES, it)
        p.dgc.dgc_set_iteration_density(it)
        p.ocfg.density = d
        say(f"[sorted speech] iteration {it} density {d}")
        p.step(S.gradient(gs, 51, 0, it, scales), it, check_state=(it == 1), label=f"sorted speech it{it}")
    p.close()


def _merge_case(gs, N, density, seed, scales=None, preset=None, flags=SORTED, **extra):
    """N payloads from correlated streams, accumulated at a density where the receive side
    merges by element range in LDS, workers in order: bit-exact against the oracle's
    ordered sum, whether the regions ascend throughout or only part by part."""
    import torch
    kw = dict(momentum=0.9, density=density, seed=seed, num_workers=N, flags=flags, **extra)
    shared = S.gradient(gs, seed, 999, 0, scales)
    pairs, payloads = [], []
    for w in range(N):
        p = Pair(gs.offsets, **kw)
        res = p.step(S.correlated_gradient(gs, seed, w, 0, shared, scales=scales), 0, check_state=False,
                     label=f"merge N={N} w{w}")
        assert not res.overflow
        p.u = p.v = None
        p.ou = p.ov = None
        payloads.append(O.flatten_payload(res))
        pairs.append(p)
    n = gs.numel
    rng = np.random.default_rng(seed)
    start = rng.standard_normal(n).astype(np.float32) if preset else np.zeros(n, np.float32)
    expect = start.copy()
    O.decompress_accumulate(expect, payloads)
    acc = B.Dgc(B.make_config(**{k: v for k, v in kw.items() if k != "layout_density"}), gs.offsets)
    acc.set_layout(pairs[0].layout)
    dense = torch.from_numpy(start).cuda()
    acc.dgc_decompress_accumulate_regions(dense, [p.out_idx for p in pairs], [p.out_val for p in pairs],
                                          [p.out_counts for p in pairs])
    got = dense.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), expect.view(np.uint32)), \
        np.flatnonzero(got.view(np.uint32) != expect.view(np.uint32))[:5]
    overlap = S.topk_overlap(payloads[0][0], payloads[-1][0]) if N > 1 else 0.0
    # the sparse clear: zero at every index of a payload, nothing else touched
    for i, _ in payloads:
        expect[i] = 0.0
    acc.dgc_dense_clear_regions(dense, [p.out_idx for p in pairs], [p.out_counts for p in pairs])
    got = dense.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), expect.view(np.uint32))
    acc.close()
    for p in pairs:
        p.close()
    return sum(i.size for i, _ in payloads), overlap


@pytest.mark.parametrize("flags", [SORTED, 0, B.DGC_FLAG_DETERMINISTIC_ACCUMULATE])
@pytest.mark.parametrize("N,density,preset", [(1, 0.001, False), (4, 0.002, True), (16, 0.001, False),
                                               (40, 0.001, True), (48, 0.005, False)])
def test_payloads_are_merged_in_worker_order(N, density, preset, flags):
    gs = S.ragged_set(22, tensors=12, max_numel=400000)
    total, overlap = _merge_case(gs, N, density, 70 + N, preset=preset, flags=flags,
                                 layout_density=max(density, 0.01) * 4, sample_min=1024, sample_max=8192)
    say(f"[merge] N={N} d={density}: {total} pairs, overlap first/last {overlap:.2f}")


@pytest.mark.parametrize("flags", [SORTED, 0])
@pytest.mark.parametrize("N,density,preset", [(1, 0.02, True), (3, 0.0625, False), (8, 0.25, True), (3, 1.0, True),
                                               (20, 0.25, False)])
def test_payloads_are_merged_part_by_part_at_warmup_densities(N, density, preset, flags):
    """Above 0.5 % the receive side keeps one emit part's range of the dense vector in LDS:
    the same bit-exact ordered sum, and the sparse clear by bitmap."""
    gs = S.ragged_set(24, tensors=12, max_numel=400000)
    total, overlap = _merge_case(gs, N, density, 170 + N, preset=preset, flags=flags, layout_density=density,
                                 sample_min=1024, sample_max=8192)
    say(f"[merge parts] N={N} d={density}: {total} pairs, overlap first/last {overlap:.2f}")


def test_part_merge_of_many_tiny_tensors():
    sizes = [1 + (7 * i) % 300 for i in range(1500)] + [40000, 3, 70001]
    gs = S.GradientSet("tiny", tuple(S.TensorSpec(f"t{i}", (s,)) for i, s in enumerate(sizes)))
    _merge_case(gs, 4, 0.1, 77, preset=True, flags=0, layout_density=0.1, sample_min=64, sample_max=512)


@pytest.mark.parametrize("flags", [SORTED, 0])
def test_sixteen_worker_merge_resnet50_shape(flags):
    gs = S.resnet50_set()
    total, overlap = _merge_case(gs, 16, 0.001, 61, scales=S.tensor_scales(gs, 61), flags=flags)
    say(f"[merge] resnet50 N=16: {total} pairs, overlap {overlap:.2f}")
    assert 0.15 < overlap < 0.5


@pytest.mark.parametrize("density,flags", [(0.002, SORTED), (0.0625, 0), (0.25, SORTED)])
def test_sparse_sgd_apply_is_merged_in_worker_order(density, flags):
    import torch
    gs = S.ragged_set(23, tensors=9, max_numel=300000)
    N, lr = 6, 0.05
    kw = dict(momentum=0.9, density=density, seed=12, num_workers=N, flags=flags, sample_min=1024, sample_max=8192)
    shared = S.gradient(gs, 29, 99, 0)
    pairs, payloads = [], []
    for w in range(N):
        p = Pair(gs.offsets, layout_density=max(0.02, density), **kw)
        res = p.step(S.correlated_gradient(gs, 29, w, 0, shared), 0, label=f"sgd d={density} w{w}")
        payloads.append(O.flatten_payload(res))
        pairs.append(p)
    rng = np.random.default_rng(5)
    theta0 = rng.standard_normal(gs.numel).astype(np.float32)
    expect = theta0.copy()
    O.sparse_sgd_apply(expect, payloads, lr)
    opt = B.Dgc(B.make_config(**kw), gs.offsets)
    opt.set_layout(pairs[0].layout)
    theta = torch.from_numpy(theta0).cuda()
    opt.dgc_sparse_sgd_apply_regions(theta, lr, [p.out_idx for p in pairs], [p.out_val for p in pairs],
                                     [p.out_counts for p in pairs])
    assert np.array_equal(theta.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    opt.close()
    for p in pairs:
        p.close()
