"""The compress and accumulate calls under HIP graph capture: the library allocates
nothing and synchronises nothing on the hot path, and every counter its kernels use is
left at zero by the kernels themselves, so a captured step can be replayed.  Every
replay is checked against the oracle, with eager work and synchronisations between the
replays.  Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import gather_payload, oracle_config, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("flags,extra,warm", [
    (0, dict(clip_threshold=0.05, num_workers=4), False),
    (B.DGC_FLAG_SORTED_OUTPUT, dict(refine_alpha=1.0, sample_min=64, sample_max=64, sample_block=4), False),
    (0, dict(), True),                  # staged streaming pass, part kernels on the receive side
])
def test_captured_step_replays_match_the_oracle(flags, extra, warm):
    import torch
    gs = S.ragged_set(19, tensors=14, max_numel=150000)
    n = gs.numel
    kw = dict(momentum=0.9, density=0.01, seed=6, flags=flags, **extra)
    dgc = B.Dgc(B.make_config(**kw), gs.offsets, warmup_workspace=warm)
    layout = dgc.dgc_recommended_payload_layout(0.05)
    dgc.set_layout(layout)
    caps = [layout[j + 1] - layout[j] for j in range(len(gs.sizes))]
    ocfg = oracle_config(**kw)
    u = torch.zeros(n, device="cuda")
    v = torch.zeros(n, device="cuda")
    g_static = torch.zeros(n, device="cuda")
    dense = torch.zeros(n, device="cuda")
    out_idx, out_val, out_counts, out_thr = dgc.alloc_payload("cuda")
    iteration = 5                                          # frozen into the captured launch arguments
    grads = [S.gradient(gs, 33, 0, it) for it in range(5)]

    # a first call inside a capture would have to upload the tables: refused, nothing enqueued
    refused = torch.cuda.CUDAGraph()
    with torch.cuda.graph(refused):
        with pytest.raises(B.DgcError) as err:
            dgc.dgc_compress(g_static, u, v, out_idx, out_val, out_counts, out_thr, iteration)
        assert err.value.status == B.DGC_ERR_STATE
        u.add_(0.0)                                        # (a capture must not be empty)
    del refused

    # first use uploads the tables (host copies): outside the capture
    g_static.copy_(torch.from_numpy(grads[4]))
    dgc.dgc_compress(g_static, u, v, out_idx, out_val, out_counts, out_thr, iteration)
    dgc.dgc_decompress_accumulate_regions(dense, [out_idx], [out_val], [out_counts])
    torch.cuda.synchronize()
    u.zero_(); v.zero_(); dense.zero_()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dgc.dgc_compress(g_static, u, v, out_idx, out_val, out_counts, out_thr, iteration)
        dgc.dgc_decompress_accumulate_regions(dense, [out_idx], [out_val], [out_counts])
    u.zero_(); v.zero_(); dense.zero_()                     # capture does not run the kernels; be explicit anyway

    ou = np.zeros(n, np.float32)
    ov = np.zeros(n, np.float32)
    expect_dense = np.zeros(n, np.float32)
    for rep in range(4):
        g_static.copy_(torch.from_numpy(grads[rep]))
        graph.replay()
        torch.cuda.synchronize()
        res = O.compress(grads[rep], ou, ov, gs.offsets, ocfg, iteration, caps)
        per_idx, per_val, counts = gather_payload(layout, out_idx, out_val, out_counts)
        diag = dgc.dgc_get_diagnostics()
        if ocfg.clip_threshold > 0:
            assert abs(diag.norm - res.norm) <= 1e-6 * res.norm
            # The captured call uses the library's own clipping scale.  Everything below is compared bit
            # for bit, which holds when that scale has the oracle's bits (it does for these seeds; a
            # reduction in another order differs in the last bit about once in 1e8 calls, and what
            # must hold then is tested in test_gpu_parity.py with a scale that is off on purpose).
            assert np.float32(diag.scale) == res.scale
        assert np.array_equal(out_thr.cpu().numpy().view(np.uint32), res.thresholds.view(np.uint32)), rep
        assert np.array_equal(counts.astype(np.int64), res.counts), rep
        assert not res.overflow
        for j in range(len(gs.sizes)):
            assert np.array_equal(per_idx[j], res.indices[j]), (rep, j)
            assert np.array_equal(per_val[j].view(np.uint32), res.values[j].view(np.uint32)), (rep, j)
        assert np.array_equal(u.cpu().numpy().view(np.uint32), ou.view(np.uint32)), rep
        assert np.array_equal(v.cpu().numpy().view(np.uint32), ov.view(np.uint32)), rep
        O.decompress_accumulate(expect_dense, [O.flatten_payload(res)])
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect_dense.view(np.uint32)), rep
        # the program's own eager work between replays
        scratch = torch.randn(100000, device="cuda")
        assert torch.isfinite(scratch.sum()).item()
        say(f"[graph] replay {rep}: {int(counts.sum())} pairs, refined {sum(res.refined)}")
    dgc.close()


def test_two_handles_alternating_on_one_workspace():
    """A workspace handed back and forth between two handles (different gradient sets, so
    different tables): every call finds the tables of its own handle, because the library
    notices the change of owner and uploads them again."""
    import torch
    sets = [S.ragged_set(5, tensors=11, max_numel=90000), S.ragged_set(6, tensors=17, max_numel=120000)]
    kws = [dict(momentum=0.9, density=0.01, seed=3), dict(momentum=0.8, density=0.02, seed=4, refine_alpha=1.5)]
    handles, layouts, states, oracles = [], [], [], []
    for gs, kw in zip(sets, kws):
        d = B.Dgc(B.make_config(**kw), gs.offsets)
        layout = d.dgc_recommended_payload_layout(0.05)
        d.set_layout(layout)
        handles.append(d)
        layouts.append(layout)
        states.append((torch.zeros(gs.numel, device="cuda"), torch.zeros(gs.numel, device="cuda"),
                       d.alloc_payload("cuda")))
        oracles.append((np.zeros(gs.numel, np.float32), np.zeros(gs.numel, np.float32), oracle_config(**kw)))
    nbytes = max(d.dgc_workspace_bytes() for d in handles)
    shared = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    for d in handles:                                       # both handles are given the same device memory
        d.workspace = shared
        d._ws_ptr = (shared.data_ptr() + 255) // 256 * 256
        d._ws_bytes = nbytes
    for it in range(3):
        for w in (0, 1, 1, 0):
            gs, d, layout = sets[w], handles[w], layouts[w]
            u, v, (out_idx, out_val, out_counts, out_thr) = states[w]
            ou, ov, ocfg = oracles[w]
            g = S.gradient(gs, 40 + w, 0, it)
            d.dgc_compress(torch.from_numpy(g).cuda(), u, v, out_idx, out_val, out_counts, out_thr, it)
            caps = [layout[j + 1] - layout[j] for j in range(len(gs.sizes))]
            res = O.compress(g, ou, ov, gs.offsets, ocfg, it, caps)
            per_idx, per_val, counts = gather_payload(layout, out_idx, out_val, out_counts)
            assert not res.overflow
            assert np.array_equal(out_thr.cpu().numpy().view(np.uint32), res.thresholds.view(np.uint32)), (it, w)
            for j in range(len(gs.sizes)):
                assert np.array_equal(per_idx[j], res.indices[j]), (it, w, j)
                assert np.array_equal(per_val[j].view(np.uint32), res.values[j].view(np.uint32)), (it, w, j)
            assert np.array_equal(v.cpu().numpy().view(np.uint32), ov.view(np.uint32)), (it, w)
            assert np.array_equal(u.cpu().numpy().view(np.uint32), ou.view(np.uint32)), (it, w)
    # the caller overwrites the workspace: announced, so the tables are uploaded again
    shared.zero_()
    handles[0].dgc_invalidate_workspace()
    gs, d, layout = sets[0], handles[0], layouts[0]
    u, v, (out_idx, out_val, out_counts, out_thr) = states[0]
    ou, ov, ocfg = oracles[0]
    g = S.gradient(gs, 40, 0, 99)
    d.dgc_compress(torch.from_numpy(g).cuda(), u, v, out_idx, out_val, out_counts, out_thr, 7)
    res = O.compress(g, ou, ov, gs.offsets, ocfg, 7, [layout[j + 1] - layout[j] for j in range(len(gs.sizes))])
    per_idx, per_val, counts = gather_payload(layout, out_idx, out_val, out_counts)
    for j in range(len(gs.sizes)):
        assert np.array_equal(per_idx[j], res.indices[j]), j
    assert np.array_equal(v.cpu().numpy().view(np.uint32), ov.view(np.uint32))
    for d in handles:
        d.close()
