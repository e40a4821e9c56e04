"""GPU parity of the wire format (32-bit values + 16-bit zero-run lengths): dgc_encode of
a sorted payload against the oracle's encode(), entry by entry, and
dgc_decode_accumulate against the oracle's decoder.  Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import Pair, say

pytestmark = pytest.mark.gpu

SORTED = B.DGC_FLAG_SORTED_OUTPUT


def encode_on_gpu(p: Pair, capacity=None):
    import torch
    pairs = sum(min(int(c), cap) for c, cap in zip(p.out_counts.cpu().tolist(), p.capacities))
    cap = p.dgc.dgc_encode_max_entries(pairs) if capacity is None else capacity
    runs = torch.full((cap + 8,), -1, dtype=torch.int16, device="cuda")
    vals = torch.full((cap + 8,), float("nan"), dtype=torch.float32, device="cuda")
    num = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    p.dgc.dgc_encode(p.out_idx, p.out_val, p.out_counts, runs[:cap], vals[:cap], num)
    e = int(num.item())
    return runs, vals, e


def check_against_oracle(p: Pair, res, label):
    runs, vals, e = encode_on_gpu(p)
    o_runs, o_vals = O.encode(*O.flatten_payload(res))
    assert e == o_runs.size, (label, e, o_runs.size)
    got_runs = runs[:e].cpu().numpy().view(np.uint16)
    got_vals = vals[:e].cpu().numpy()
    assert np.array_equal(got_runs, o_runs), (label, "runs")
    assert np.array_equal(got_vals.view(np.uint32), o_vals.view(np.uint32)), (label, "values")
    assert not (p.dgc.dgc_get_diagnostics().flags & (B.DGC_DIAG_UNSORTED | B.DGC_DIAG_OVERFLOW))
    return runs, vals, e


def test_encode_ragged_set_and_decode_round_trip():
    import torch
    gs = S.ragged_set(3)
    N = 3
    kw = dict(layout_density=0.05, momentum=0.9, density=0.01, seed=11, sample_min=256, sample_max=2048,
              flags=SORTED)
    pairs = [Pair(gs.offsets, **kw) for _ in range(N)]
    shared = S.gradient(gs, 40, 99, 0)
    for it in range(2):
        enc, oracle_entries = [], []
        for w, p in enumerate(pairs):
            res = p.step(S.correlated_gradient(gs, 40, w, it, shared), it, label=f"wire w{w} it{it}")
            runs, vals, e = check_against_oracle(p, res, f"wire w{w} it{it}")
            enc.append((runs, vals, e))
            oracle_entries.append(O.encode(*O.flatten_payload(res)))
        expect = np.zeros(gs.numel, np.float32)
        for r, x in oracle_entries:
            O.decode_accumulate(expect, r, x)
        cfg_kw = {k: v for k, v in kw.items() if k != "layout_density"}
        det = B.Dgc(B.make_config(**{**cfg_kw, "flags": SORTED | B.DGC_FLAG_DETERMINISTIC_ACCUMULATE}), gs.offsets)
        dense = torch.zeros(gs.numel, device="cuda")
        det.dgc_decode_accumulate(dense, [r for r, _, _ in enc], [x for _, x, _ in enc], [e for _, _, e in enc])
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
        dense.zero_()
        pairs[0].dgc.dgc_decode_accumulate(dense, [r for r, _, _ in enc], [x for _, x, _ in enc],
                                           [e for _, _, e in enc])
        mags = np.zeros(gs.numel, np.float64)
        for p in pairs:
            i, x = O.flatten_payload(p.last[0])
            np.add.at(mags, i.astype(np.int64), np.abs(x.astype(np.float64)))
        assert np.all(np.abs(dense.cpu().numpy().astype(np.float64) - expect) <= 1e-6 * mags)
        det.close()
    for p in pairs:
        p.close()


def test_encode_long_gaps_need_filler_entries():
    import torch
    # three tensors, almost everything zero: gaps of more than 65535 zeros inside a tensor,
    # across a tensor boundary, across an empty region, and of exactly 65535 and 65536
    sizes = [300000, 40, 70000, 200000, 131072 + 5]
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    n = int(offsets[-1])
    p = Pair(offsets, layout_density=0.01, momentum=0.0, density=0.001, seed=2, flags=SORTED | B.DGC_FLAG_EXACT_SELECT)
    g = np.zeros(n, np.float32)
    hot = [5, 5 + 65536, 5 + 65536 + 65537, 299999,                       # gaps 65535, 65536, long
           int(offsets[3]) + 150000,                                        # regions 1 and 2 stay empty
           int(offsets[4]) + 3, int(offsets[4]) + 3 + 131072]               # two fillers then run 0 ... exact multiple
    g[hot] = np.arange(1, len(hot) + 1, dtype=np.float32) * np.float32(-1.5)
    res = p.step(g, 0, label="long gaps")
    assert sorted(O.flatten_payload(res)[0].tolist()) == sorted(hot)      # thr = 0: only the non-zeros pass
    runs, vals, e = check_against_oracle(p, res, "long gaps")
    o_runs, _ = O.encode(*O.flatten_payload(res))
    assert e > len(hot) and int((o_runs == 65535).sum()) >= 4
    dense = torch.zeros(n, device="cuda")
    p.dgc.dgc_decode_accumulate(dense, [runs], [vals], [e])
    assert np.array_equal(dense.cpu().numpy(), g)
    # a capacity that is too small drops the tail and raises the flag, without writing past it
    small = e - 2
    runs2, vals2, e2 = encode_on_gpu(p, capacity=small)
    assert e2 == e
    assert p.dgc.dgc_get_diagnostics().flags & B.DGC_DIAG_OVERFLOW
    assert np.array_equal(runs2[:small].cpu().numpy(), runs[:small].cpu().numpy())
    assert int(runs2[small].item()) == -1 and np.isnan(vals2[small].item())
    p.close()


def test_encode_flags_an_unsorted_region_and_decode_flags_a_bad_position():
    import torch
    n = 50000
    p = Pair([0, n], layout_density=0.01, momentum=0.0, density=0.002, seed=3)     # not sorted
    rng = np.random.default_rng(8)
    p.step(rng.standard_normal(n).astype(np.float32), 0, label="unsorted source")
    idx = p.out_idx.cpu().numpy()[: int(p.out_counts.item())]
    if np.all(np.diff(idx) > 0):                                                      # arrival order happened to be ascending
        p.out_idx[:2] = p.out_idx[:2].flip(0)
    encode_on_gpu(p)
    assert p.dgc.dgc_get_diagnostics().flags & B.DGC_DIAG_UNSORTED
    dense = torch.zeros(100, device="cuda")
    runs = torch.tensor([3, 90, 20], dtype=torch.int16, device="cuda")
    vals = torch.tensor([1.0, 2.0, 3.0], dtype=torch.float32, device="cuda")
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    small = B.Dgc(B.dgc_config_default(), [0, 100])
    small.dgc_decode_accumulate(dense, [runs], [vals], [3], diag_flags=flags)
    out = dense.cpu().numpy()
    assert out[3] == 1.0 and out[94] == 2.0 and out.sum() == 3.0
    assert int(flags.item()) & B.DGC_DIAG_BAD_INDEX
    small.dgc_decode_accumulate(dense, [runs, runs], [vals, vals], [0, 0])           # empty payloads
    assert dense.cpu().numpy().sum() == 3.0
    small.close()
    p.close()


def test_encode_resnet50_set_and_sixteen_payload_decode():
    import torch
    gs = S.resnet50_set()
    N = 4
    scales = S.tensor_scales(gs, 61)
    shared = S.gradient(gs, 61, 999, 0, scales)
    kw = dict(momentum=0.9, density=0.001, seed=61, num_workers=N, flags=SORTED)
    enc, payloads, keep = [], [], []
    for w in range(N):
        p = Pair(gs.offsets, **kw)
        res = p.step(S.correlated_gradient(gs, 61, w, 0, shared, scales=scales), 0, check_state=False,
                     label=f"wire resnet w{w}")
        runs, vals, e = check_against_oracle(p, res, f"wire resnet w{w}")
        pairs_w = int(res.counts.sum())
        say(f"[wire] worker {w}: {pairs_w} pairs -> {e} entries, {O.encoded_bytes(e)} bytes, "
            f"ratio {4.0 * gs.numel / O.encoded_bytes(e):.0f}x (paper, Table 3: 277x)")
        enc.append((runs, vals, e))
        payloads.append(O.flatten_payload(res))
        p.u = p.v = None
        keep.append(p)
    expect = np.zeros(gs.numel, np.float32)
    O.decompress_accumulate(expect, payloads)          # the decoder must give what the pair lists give
    det = B.Dgc(B.make_config(**{**kw, "flags": SORTED | B.DGC_FLAG_DETERMINISTIC_ACCUMULATE}), gs.offsets)
    dense = torch.zeros(gs.numel, device="cuda")
    det.dgc_decode_accumulate(dense, [r for r, _, _ in enc], [x for _, x, _ in enc], [e for _, _, e in enc])
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    for p in keep:
        p.close()


def test_thousands_of_tiny_tensors_through_every_pass():
    # more tensors than a tile has lanes, than the receive side stages at a time, and than
    # the encoder looks back at once: 1-element tensors by the hundred inside one tile
    import torch
    rng = np.random.default_rng(17)
    sizes = [1] * 1500 + [3] * 700 + [5000] + [2] * 900 + [70000] + [1] * 130 + [7]
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    n = int(offsets[-1])
    T = len(sizes)
    kw = dict(layout_density=1.0, momentum=0.9, density=0.02, seed=4, sample_min=64, sample_max=256,
              flags=SORTED)
    workers = [Pair(offsets, **kw) for _ in range(2)]
    enc, oracle_entries, payloads = [], [], []
    for it in range(2):
        enc, oracle_entries, payloads = [], [], []
        for w, p in enumerate(workers):
            g = rng.standard_t(3, n).astype(np.float32)
            g[rng.random(n) < 0.5] = 0.0                       # many tensors send nothing at all
            res = p.step(g, it, label=f"tiny tensors w{w} it{it}")
            runs, vals, e = check_against_oracle(p, res, f"tiny tensors w{w} it{it}")
            enc.append((runs, vals, e))
            oracle_entries.append(O.encode(*O.flatten_payload(res)))
            payloads.append(O.flatten_payload(res))
    expect = np.zeros(n, np.float32)
    O.decompress_accumulate(expect, payloads)
    cfg_kw = {k: v for k, v in kw.items() if k != "layout_density"}
    det = B.Dgc(B.make_config(**{**cfg_kw, "flags": SORTED | B.DGC_FLAG_DETERMINISTIC_ACCUMULATE}), offsets)
    det.set_layout(workers[0].layout)
    dense = torch.zeros(n, device="cuda")
    det.dgc_decompress_accumulate_regions(dense, [p.out_idx for p in workers], [p.out_val for p in workers],
                                          [p.out_counts for p in workers])
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    dense.zero_()
    det.dgc_decode_accumulate(dense, [r for r, _, _ in enc], [x for _, x, _ in enc], [e for _, _, e in enc])
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
    det.dgc_dense_clear_regions(dense, [p.out_idx for p in workers], [p.out_counts for p in workers])
    assert not dense.cpu().numpy().any()
    det.close()
    for p in workers:
        p.close()
