"""dgc_compress_static, the entry point for callers that cannot allocate: its results against
those of dgc_compress (same kernels, a workspace of the caller's), on calls in a row that share
the library's static scratch array -- a larger gradient set, then a smaller one, then the first
again.  Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from paper_1712_01887_amd import binding as B
from paper_1712_01887_amd import synthetic as S
from tests.parity import say

pytestmark = pytest.mark.gpu


class Side:
    """One handle with its own state and payload buffers."""

    def __init__(self, gs, kw, layout_density):
        import torch
        self.dgc = B.Dgc(B.make_config(**kw), gs.offsets)
        self.layout = self.dgc.dgc_recommended_payload_layout(layout_density)
        self.dgc.set_layout(self.layout)
        self.u = torch.zeros(gs.numel, device="cuda")
        self.v = torch.zeros(gs.numel, device="cuda")
        self.out = self.dgc.alloc_payload("cuda")

    def outputs(self):
        idx, val, cnt, thr = (t.cpu().numpy() for t in self.out)
        pairs = []
        for j in range(len(self.layout) - 1):
            lo = self.layout[j]
            c = min(int(cnt[j]), self.layout[j + 1] - lo)
            pairs.append((idx[lo:lo + c].copy(), val[lo:lo + c].copy()))   # as the library left them: same kernels, same order
        return pairs, cnt.copy(), thr.copy(), self.u.cpu().numpy(), self.v.cpu().numpy()


def same(a, b, what):
    pa, ca, ta, ua, va = a
    pb, cb, tb, ub, vb = b
    assert np.array_equal(ca, cb), (what, "counts")
    assert np.array_equal(ta.view(np.uint32), tb.view(np.uint32)), (what, "thresholds")
    for j, ((ia, xa), (ib, xb)) in enumerate(zip(pa, pb)):
        assert np.array_equal(ia, ib), (what, "indices", j)
        assert np.array_equal(xa.view(np.uint32), xb.view(np.uint32)), (what, "values", j)
    assert np.array_equal(ua.view(np.uint32), ub.view(np.uint32)), (what, "u")
    assert np.array_equal(va.view(np.uint32), vb.view(np.uint32)), (what, "v")


def test_static_scratch_matches_the_workspace_entry_point():
    import torch
    assert torch.cuda.is_available()
    big = S.GradientSet("big", tuple(S.TensorSpec(f"t{i}", (s,)) for i, s in
                                     enumerate([1500000, 29, 640000, 4097, 3, 260000, 1024 * 70 + 1])))
    small = S.ragged_set(21, tensors=12, max_numel=60000)
    cases = [
        ("big", big, dict(momentum=0.9, density=0.001, seed=5, clip_threshold=0.05, num_workers=4), 0.004),
        ("small", small, dict(momentum=0.8, density=0.01, seed=6, refine_alpha=1.5, sample_min=256, sample_max=1024), 0.05),
    ]
    sides = {}
    for name, gs, kw, ld in cases:
        sides[name] = (gs, Side(gs, kw, ld), Side(gs, kw, ld))          # (set, static side, workspace side)
    order = ["big", "small", "big", "small", "small", "big"]             # the array changes hands between calls
    iteration = {"big": 0, "small": 0}
    for step, name in enumerate(order):
        gs, st, ws = sides[name]
        it = iteration[name]
        iteration[name] += 1
        g = torch.from_numpy(S.gradient(gs, 70 + len(name), 0, it)).cuda()
        say(f"[no-alloc] call {step}: {name} set, {gs.numel} elements, iteration {it}")
        st.dgc.dgc_compress_static(g, st.u, st.v, *st.out, it)
        ws.dgc.dgc_compress(g, ws.u, ws.v, *ws.out, it)
        torch.cuda.synchronize()
        same(st.outputs(), ws.outputs(), f"call {step} ({name})")
        ds, dw = st.dgc.dgc_get_diagnostics(static=True), ws.dgc.dgc_get_diagnostics()
        assert ds.flags == dw.flags and np.float32(ds.scale) == np.float32(dw.scale)
        assert (ds.norm == dw.norm) or (ds.norm != ds.norm and dw.norm != dw.norm)
    # a set whose workspace does not fit the array is refused, with nothing enqueued
    speech = S.speech_set()
    d = B.Dgc(B.dgc_config_default(), speech.offsets)
    d.set_layout(d.dgc_recommended_payload_layout(0.001))
    assert d.dgc_workspace_bytes() > 8 << 20
    with pytest.raises(B.DgcError) as err:
        d.dgc_compress_static(sides["big"][1].u, sides["big"][1].u, sides["big"][1].v, *sides["big"][1].out, 0)
    assert err.value.status == B.DGC_ERR_CAPACITY
    d.close()
    for _, a, b in sides.values():
        a.dgc.close()
        b.dgc.close()
