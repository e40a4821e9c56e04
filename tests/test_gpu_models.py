"""GPU parity at the full sizes of the paper-shaped gradient sets (ResNet-50,
LSTM language model, speech model) and of the 16-worker receive side.
Element-by-element against the oracle; run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import Pair, say

pytestmark = pytest.mark.gpu


def test_resnet50_set_ten_iterations():
    gs = S.resnet50_set()
    scales = S.tensor_scales(gs, 31)
    p = Pair(gs.offsets, momentum=0.9, density=0.001, seed=31)
    total = 0
    for it in range(10):
        say(f"[resnet50] iteration {it}")
        res = p.step(S.gradient(gs, 31, 0, it, scales), it, label=f"resnet50 it{it}")
        total = int(res.counts.sum())
        # 108 of the 161 tensors are small enough to be selected exactly
        for j, n in enumerate(gs.sizes):
            if n <= 4096:
                assert int(res.counts[j]) == O.topk_count(0.001, n)
    ratio8 = O.compression_ratio(gs.numel, total, 8)
    ratio6 = O.compression_ratio(gs.numel, total, 6)
    say(f"[resnet50] pairs={total} ratio(8 B/pair)={ratio8:.0f}x ratio(6 B/pair)={ratio6:.0f}x "
        f"(paper, Table 3: 277x)")
    assert 0.5 * 25670 < total < 2.0 * 25670
    p.close()


def test_resnet50_set_with_rethreshold():
    gs = S.resnet50_set()
    scales = S.tensor_scales(gs, 32)
    p = Pair(gs.offsets, momentum=0.9, density=0.001, seed=32, refine_alpha=2.0)
    for it in range(2):
        res = p.step(S.gradient(gs, 32, 0, it, scales), it, label=f"resnet50 refine it{it}")
        say(f"[resnet50 refine] iteration {it}: {sum(res.refined)} tensors re-thresholded, pairs={int(res.counts.sum())}")
        assert not res.overflow
        for j, n in enumerate(gs.sizes):
            assert int(res.counts[j]) <= 2 * O.topk_count(0.001, n)
    p.close()


def test_lstm_set_with_clipping_two_iterations():
    gs = S.lstm_lm_set()
    scales = S.tensor_scales(gs, 41)
    p = Pair(gs.offsets, momentum=0.9, density=0.001, seed=41, clip_threshold=0.25, num_workers=4)
    for it in range(2):
        say(f"[lstm] iteration {it}")
        res = p.step(S.lstm_gradient(gs, 41, 0, it, scales), it, label=f"lstm it{it}")
        say(f"[lstm] norm={res.norm:.4f} scale={float(res.scale):.6f} embedding pairs={int(res.counts[0])}")
    p.close()


def test_speech_set_warmup_schedule_twenty_iterations():
    """The whole configuration: densities 25 %, 6.25 %, 1.5625 %, 0.4 %, then 0.1 % held to iteration
    19 (Section 4.1's sparsities), one worker of N = 8; thresholds, index sets and values of every
    iteration, u and v at the ends of the ramp and of the run."""
    gs = S.speech_set()
    scales = S.tensor_scales(gs, 51)
    p = Pair(gs.offsets, layout_density=0.25, momentum=0.9, density=0.25, seed=51, num_workers=8)
    for it in range(20):
        d = O.warmup_density(O.WARMUP_DENSITIES, it)
        p.dgc.dgc_set_iteration_density(it)
        p.ocfg.density = d
        say(f"[speech] iteration {it} density {d}")
        res = p.step(S.gradient(gs, 51, 0, it, scales), it, check_state=(it in (0, 4, 5, 19)),
                     label=f"speech it{it}")
        say(f"[speech] pairs={int(res.counts.sum())} expected~{int(d * gs.numel)}")
    p.close()


def test_speech_set_receive_side_eight_workers():
    """The receive side at the speech set's full size with N = 8: a warm-up density (6.25 %), then the
    steady state (0.1 %) twice, so that the replacing merge runs both after a warm-up iteration (the
    whole aggregate is rewritten) and after a steady-state one (only the previous and the new
    indices are touched).  Accumulate, sparse clear and replace, bit for bit against the oracle's sum
    with the workers added in order."""
    import torch
    gs = S.speech_set()
    scales = S.tensor_scales(gs, 58)
    N = 8
    kw = dict(momentum=0.9, density=0.0625, seed=58, num_workers=N)
    shared = S.gradient(gs, 58, 999, 0, scales)
    grads = [S.correlated_gradient(gs, 58, w, 0, shared, scales=scales) for w in range(N)]
    del shared
    pairs = [Pair(gs.offsets, layout_density=0.0625, **kw) for _ in range(N)]
    acc = B.Dgc(B.make_config(**kw), gs.offsets)
    acc.set_layout(pairs[0].layout)
    dense = torch.zeros(gs.numel, device="cuda")
    previous = None
    for it, d in enumerate([0.0625, 0.001, 0.001]):
        payloads = []
        for w, p in enumerate(pairs):
            p.set_density(d)
            say(f"[speech N=8] iteration {it} density {d} worker {w}")
            res = p.step(grads[w], it, check_state=False, label=f"speech N=8 it{it} w{w}")
            assert not res.overflow
            payloads.append(O.flatten_payload(res))
        expect = np.zeros(gs.numel, np.float32)
        O.decompress_accumulate(expect, payloads)
        lists = ([p.out_idx for p in pairs], [p.out_val for p in pairs], [p.out_counts for p in pairs])
        acc.dgc_set_density(d)
        if previous is None:
            acc.dgc_decompress_accumulate_regions(dense, *lists)
            assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32)), "accumulate"
            acc.dgc_dense_clear_regions(dense, lists[0], lists[2])
            assert not dense.any().item(), "sparse clear"
            acc.dgc_decompress_replace_regions(dense, *lists)
        else:
            acc.dgc_decompress_replace_regions(dense, *lists, previous[0], previous[1])
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32)), f"replace it{it}"
        if it == 2:                                      # and the two-call way at 0.1 %, from a zero buffer
            scratch = torch.zeros(gs.numel, device="cuda")
            acc.dgc_decompress_accumulate_regions(scratch, *lists)
            assert np.array_equal(scratch.cpu().numpy().view(np.uint32), expect.view(np.uint32)), "accumulate 0.1 %"
            acc.dgc_dense_clear_regions(scratch, lists[0], lists[2])
            assert not scratch.any().item(), "sparse clear 0.1 %"
            del scratch
        # the next iteration overwrites the workers' payload buffers: keep this one's index lists
        previous = ([p.out_idx.clone() for p in pairs], [p.out_counts.clone() for p in pairs])
    acc.close()
    for p in pairs:
        p.close()


def test_literal_speech_set_two_iterations():
    """The 90 M-element set of five bidirectional GRU-1024 layers: a warm-up step with the
    staging workspace, then the steady state."""
    gs = S.speech_literal_set()
    scales = S.tensor_scales(gs, 53)
    p = Pair(gs.offsets, warmup_workspace=True, layout_density=0.0625, momentum=0.9, density=0.0625, seed=53,
             num_workers=8)
    for it, d in enumerate([0.0625, 0.001]):
        p.set_density(d)
        say(f"[speech literal] iteration {it} density {d}")
        p.step(S.gradient(gs, 53, 0, it, scales), it, check_state=(it == 1), label=f"speech literal it{it}")
    p.close()


def test_speech_set_receive_side_at_warmup_densities():
    """The receive side above 0.5 % at the speech set's full size (3764 emit parts: every
    workgroup of the part kernels takes several), two workers: accumulate, sparse clear and
    the replacing merge against the oracle's ordered sum, bit for bit."""
    import torch
    gs = S.speech_set()
    scales = S.tensor_scales(gs, 57)
    N = 2
    kw = dict(momentum=0.9, density=0.25, seed=57, num_workers=N)
    shared = S.gradient(gs, 57, 999, 0, scales)
    pairs = [Pair(gs.offsets, warmup_workspace=True, layout_density=0.0625, **kw) for _ in range(N)]
    acc = B.Dgc(B.make_config(**kw), gs.offsets)
    acc.set_layout(pairs[0].layout)
    dense = torch.zeros(gs.numel, device="cuda")
    for it, d in enumerate([0.25, 0.0625]):
        payloads = []
        for w, p in enumerate(pairs):
            p.set_density(d)
            say(f"[speech receive] iteration {it} density {d} worker {w}")
            res = p.step(S.correlated_gradient(gs, 57, w, it, shared, scales=scales), it, check_state=False,
                         label=f"speech receive it{it} w{w}")
            assert not res.overflow
            payloads.append(O.flatten_payload(res))
        expect = np.zeros(gs.numel, np.float32)
        O.decompress_accumulate(expect, payloads)
        lists = ([p.out_idx for p in pairs], [p.out_val for p in pairs], [p.out_counts for p in pairs])
        acc.dgc_set_density(d)
        if it == 0:
            acc.dgc_decompress_accumulate_regions(dense, *lists)
            assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32)), "accumulate"
            acc.dgc_dense_clear_regions(dense, lists[0], lists[2])
            assert not dense.any().item(), "sparse clear"
            acc.dgc_decompress_replace_regions(dense, *lists)
        else:                                            # over the aggregate of iteration 0, whose lists are gone
            acc.dgc_decompress_replace_regions(dense, *lists)
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32)), f"replace it{it}"
    acc.close()
    for p in pairs:
        p.close()


def test_sixteen_worker_accumulate_resnet50_shape():
    import torch
    gs = S.resnet50_set()
    N = 16
    scales = S.tensor_scales(gs, 61)
    shared = S.gradient(gs, 61, 999, 0, scales)
    kw = dict(momentum=0.9, density=0.001, seed=61, num_workers=N)
    pairs = []
    payloads = []
    for w in range(N):
        say(f"[accumulate] worker {w}")
        p = Pair(gs.offsets, **kw)
        res = p.step(S.correlated_gradient(gs, 61, w, 0, shared, scales=scales), 0, check_state=False,
                     label=f"acc w{w}")
        assert not res.overflow                          # else which pairs were kept is order-dependent
        p.u = p.v = None                                 # keep only the payload on the device
        p.ou = p.ov = None
        payloads.append(O.flatten_payload(res))
        pairs.append(p)
    overlap = S.topk_overlap(payloads[0][0], payloads[1][0])
    say(f"[accumulate] pairs/worker ~{payloads[0][0].size}, pairwise index overlap {overlap:.2f}")
    assert 0.15 < overlap < 0.5
    expect = np.zeros(gs.numel, np.float32)
    O.decompress_accumulate(expect, payloads)
    torch.cuda.empty_cache()
    acc = B.Dgc(B.make_config(**kw), gs.offsets)
    acc.set_layout(pairs[0].layout)
    dense = torch.zeros(gs.numel, dtype=torch.float32, device="cuda")
    idx = [p.out_idx for p in pairs]
    val = [p.out_val for p in pairs]
    cnt = [p.out_counts for p in pairs]
    acc.dgc_decompress_accumulate_regions(dense, idx, val, cnt)
    got = dense.cpu().numpy()
    # Summing N binary32 terms in any order stays within (N-1) * 2**-24 * sum|x| of the exact sum
    # (15 * 2**-24 = 8.9e-7 < 1e-6 for N = 16).  The oracle's worker-ordered sum obeys the same
    # bound, so the two may differ by up to twice that.
    mags = np.zeros(gs.numel, np.float32)
    O.decompress_accumulate(mags, [(i, np.abs(x)) for i, x in payloads])
    exact = np.zeros(gs.numel, np.float64)
    for i, x in payloads:
        np.add.at(exact, i.astype(np.int64), x.astype(np.float64))
    touched = mags > 0
    err_exact = np.abs(got.astype(np.float64) - exact)[touched] / mags[touched]
    err_oracle = np.abs(got.astype(np.float64) - expect)[touched] / mags[touched]
    say(f"[accumulate] max error / sum|x|: vs exact {err_exact.max():.3e}, vs oracle {err_oracle.max():.3e}")
    assert err_exact.max() <= 1e-6
    assert err_oracle.max() <= 2e-6
    assert not got[~touched].any()
    det = B.Dgc(B.make_config(flags=B.DGC_FLAG_DETERMINISTIC_ACCUMULATE, **kw), gs.offsets)
    det.set_layout(pairs[0].layout)
    dense.zero_()
    det.dgc_decompress_accumulate_regions(dense, idx, val, cnt)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    acc.dgc_dense_clear_regions(dense, idx, cnt)
    assert int(torch.count_nonzero(dense).item()) == 0
    for p in pairs:
        p.close()
