"""GPU parity of dgc_compress with the warm-up workspace (dgc_workspace_bytes_warmup): above a
density of 0.5 % the streaming pass masks u and v itself and parks the selected values in
staging arrays.  Every result (thresholds, index sets, values, u, v, counts, the overflow
flag) must be what the oracle computes, bit for bit, exactly as with the small workspace;
the regions come out in ascending index order whether or not the flag asks for it.
Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import Pair, check_overflow_invariants, say

pytestmark = pytest.mark.gpu

SORTED = B.DGC_FLAG_SORTED_OUTPUT


@pytest.mark.parametrize("flags", [0, SORTED, B.DGC_FLAG_NESTEROV | B.DGC_FLAG_NO_FACTOR_MASKING,
                                   B.DGC_FLAG_EXACT_SELECT | B.DGC_FLAG_NESTEROV])
@pytest.mark.parametrize("density", [0.01, 0.0625, 0.25, 1.0])
def test_staged_ragged_set(flags, density):
    gs = S.ragged_set(31)
    p = Pair(gs.offsets, warmup_workspace=True, momentum=0.9, density=density, flags=flags, seed=13,
             sample_min=256, sample_max=2048, sample_block=16)
    for it in range(3):
        p.step(S.gradient(gs, 41, 0, it), it, label=f"staged ragged flags={flags} d={density} it{it}")
    if not flags & SORTED:                                    # ascending all the same
        idx = p.out_idx.cpu().numpy()
        cnt = p.out_counts.cpu().numpy()
        for j in range(p.T):
            r = idx[p.layout[j]:p.layout[j] + min(int(cnt[j]), p.capacities[j])]
            assert np.all(np.diff(r) > 0)
    p.close()


def test_staged_edge_sizes():
    for sizes in ([1], [1023], [1024], [1025], [4096, 3], [5, 1019, 1, 2047, 7], [32768, 32769, 1, 65536],
                  [1024, 1024, 2048], [3000, 1096, 1024, 5]):
        offsets = np.concatenate([[0], np.cumsum(sizes)])
        p = Pair(offsets, warmup_workspace=True, layout_density=1.0, momentum=0.9, density=0.3, seed=1,
                 sample_min=64, sample_max=256)
        rng = np.random.default_rng(sum(sizes))
        for it in range(2):
            p.step(rng.standard_normal(offsets[-1]).astype(np.float32), it, label=f"staged sizes={sizes} it{it}")
        p.close()


def test_staged_with_clipping_and_workers():
    gs = S.ragged_set(32, tensors=18, max_numel=200000)
    p = Pair(gs.offsets, warmup_workspace=True, momentum=0.9, density=0.0625, seed=3, clip_threshold=0.25,
             num_workers=4, sample_min=512, sample_max=4096)
    for it in range(3):
        p.step(S.gradient(gs, 43, 0, it), it, label=f"staged clip it{it}")
    p.close()


@pytest.mark.parametrize("flags", [SORTED | B.DGC_FLAG_EXACT_SELECT,
                                   SORTED | B.DGC_FLAG_EXACT_SELECT | B.DGC_FLAG_NO_FACTOR_MASKING])
def test_staged_overflow_puts_elements_back_like_the_oracle(flags):
    """A full region: what does not fit goes back into v (and u), bit for bit, and passes
    again in the next iteration."""
    gs = S.ragged_set(33, tensors=10, max_numel=150000)
    caps = [max(1, O.topk_count(0.05, s) // 2) for s in gs.sizes]
    p = Pair(gs.offsets, warmup_workspace=True, capacities=caps, momentum=0.9, density=0.05, seed=9, flags=flags)
    u0 = (0.1 * S.gradient(gs, 23, 1, 0)).astype(np.float32)
    v0 = (0.1 * S.gradient(gs, 23, 2, 0)).astype(np.float32)
    p.set_state(u0, v0)
    for it in range(3):
        res = p.step(S.gradient(gs, 23, 0, it), it, label=f"staged overflow flags={flags} it{it}")
        assert res.overflow
    p.close()


def test_staged_overflow_invariants_without_the_sorted_flag():
    gs = S.ragged_set(34, tensors=10, max_numel=150000)
    caps = [max(1, O.topk_count(0.02, s) // 3) for s in gs.sizes]
    p = Pair(gs.offsets, warmup_workspace=True, capacities=caps, momentum=0.9, density=0.02, seed=19)
    u0 = (0.1 * S.gradient(gs, 27, 1, 0)).astype(np.float32)
    v0 = (0.1 * S.gradient(gs, 27, 2, 0)).astype(np.float32)
    p.set_state(u0, v0)
    g = S.gradient(gs, 27, 0, 0)
    res = p.step(g, 0, label="staged overflow, unsorted flag")
    assert res.overflow
    check_overflow_invariants(p, g, u0, v0)
    p.close()


def test_staged_rethreshold_keeps_the_plain_pass():
    gs = S.ragged_set(35, tensors=14, max_numel=120000)
    p = Pair(gs.offsets, warmup_workspace=True, momentum=0.9, density=0.01, seed=21, sample_min=64, sample_max=64,
             sample_block=4, refine_alpha=1.0)
    refined = 0
    for it in range(3):
        res = p.step(S.gradient(gs, 26, 0, it), it, label=f"staged refine it{it}")
        refined += sum(res.refined)
    assert refined >= 2
    p.close()


def test_staged_many_tiny_tensors():
    sizes = [1 + (7 * i) % 300 for i in range(1500)] + [40000, 3, 70001]
    gs = S.GradientSet("tiny", tuple(S.TensorSpec(f"t{i}", (s,)) for i, s in enumerate(sizes)))
    p = Pair(gs.offsets, warmup_workspace=True, momentum=0.9, density=0.1, seed=5, sample_min=64, sample_max=512)
    for it in range(2):
        p.step(S.gradient(gs, 45, 0, it), it, label=f"staged tiny it{it}")
    p.close()


def test_staged_warmup_schedule_on_the_speech_set():
    """25 % -> 6.25 % -> 1.5625 % -> 0.4 % -> 0.1 % in one handle and one workspace: the first
    three iterations take the staged pass, the others the plain one, on the same state."""
    gs = S.speech_set()
    scales = S.tensor_scales(gs, 52)
    p = Pair(gs.offsets, warmup_workspace=True, layout_density=0.25, momentum=0.9, density=0.25, seed=52,
             num_workers=8)
    for it in range(5):
        d = O.warmup_density(O.WARMUP_DENSITIES, it)
        p.dgc.dgc_set_iteration_density(it)
        p.ocfg.density = d
        say(f"[staged speech] iteration {it} density {d}")
        p.step(S.gradient(gs, 52, 0, it, scales), it, check_state=(it in (0, 2, 4)), label=f"staged speech it{it}")
    p.close()


def test_staged_payloads_merge_in_worker_order():
    import torch
    gs = S.ragged_set(36, tensors=12, max_numel=400000)
    N, density = 5, 0.0625
    kw = dict(momentum=0.9, density=density, seed=77, num_workers=N, sample_min=1024, sample_max=8192)
    shared = S.gradient(gs, 77, 999, 0)
    pairs, payloads = [], []
    for w in range(N):
        p = Pair(gs.offsets, warmup_workspace=True, **kw)
        res = p.step(S.correlated_gradient(gs, 77, w, 0, shared), 0, check_state=False, label=f"staged merge w{w}")
        payloads.append(O.flatten_payload(res))
        pairs.append(p)
    rng = np.random.default_rng(7)
    start = rng.standard_normal(gs.numel).astype(np.float32)
    expect = start.copy()
    O.decompress_accumulate(expect, payloads)
    acc = B.Dgc(B.make_config(**kw), gs.offsets)
    acc.set_layout(pairs[0].layout)
    dense = torch.from_numpy(start).cuda()
    acc.dgc_decompress_accumulate_regions(dense, [p.out_idx for p in pairs], [p.out_val for p in pairs],
                                          [p.out_counts for p in pairs])
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    acc.close()
    for p in pairs:
        p.close()
