"""Harness shared by the GPU parity tests: drives the HIP library and the CPU
oracle with the same seeded inputs and compares them element by element.

The oracle never sees a value computed on the GPU.

Comparison bar
  * no clipping: thresholds, per-tensor index sets, sent values, u and v bit-exact;
  * clipping on (the scale comes from a reduction, whose summation order differs between
    the two sides), two library runs per iteration from the same device state:
      (own)      the library on its own norm and scale: norm and scale within 1e-6 relative
                 of the oracle's; where the two binary32 scales are equal everything is
                 bit-exact; where they differ, sent values within 1e-6 relative, and the index
                 sets may differ only at elements whose |v'| lies within one unit in the last
                 place of the tensor's threshold, widened by how far a last-bit change of the
                 scale can move that element and the threshold (`flip_allowance`);
      (injected) the library given the ORACLE's binary32 scale: everything bit-exact.  This
                 run's state is the one the next iteration starts from.
Payload order inside a tensor's region is unspecified, so pairs are compared
after sorting by index; with DGC_FLAG_SORTED_OUTPUT the regions are compared as
the library left them, and a full region must hold the lowest indices, as in
the oracle.
"""

from __future__ import annotations

import sys

import numpy as np

from oracle import dgc_oracle as O
from paper_1712_01887_amd import binding as B


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def oracle_config(**kw) -> O.OracleConfig:
    flags = kw.pop("flags", 0)
    c = O.OracleConfig(**kw)
    c.nesterov = bool(flags & B.DGC_FLAG_NESTEROV)
    c.factor_masking = not bool(flags & B.DGC_FLAG_NO_FACTOR_MASKING)
    c.exact_select = bool(flags & B.DGC_FLAG_EXACT_SELECT)
    return c


def gather_payload(layout, out_idx, out_val, out_counts, sort: bool = True):
    """Host copy of a region-layout payload as per-tensor (indices, values), sorted by index
    unless `sort` is false (then in the order the library left them).  Waits for the device."""
    cnt = out_counts.cpu().numpy()
    used = sum(min(int(cnt[j]), layout[j + 1] - layout[j]) for j in range(len(layout) - 1))
    whole = 4 * used >= layout[-1] or len(layout) > 200    # else copy region by region (regions laid out for 25 %)
    if whole:
        idx = out_idx.cpu().numpy()
        val = out_val.cpu().numpy()
    per_idx, per_val = [], []
    for j in range(len(layout) - 1):
        lo = layout[j]
        c = min(int(cnt[j]), layout[j + 1] - lo)
        i = idx[lo:lo + c] if whole else out_idx[lo:lo + c].cpu().numpy()
        x = val[lo:lo + c] if whole else out_val[lo:lo + c].cpu().numpy()
        order = np.argsort(i, kind="stable") if sort else np.arange(c)
        per_idx.append(i[order].copy())
        per_val.append(x[order].copy())
    return per_idx, per_val, cnt


def scale_reach(gs, u1, v1, nesterov=False):
    """How far a last-bit change of the clipping scale (relative change <= 2**-23) can move v'.

    Algorithm 3: gs = fl(g * scale) moves by at most 2**-22 |gs| (the change of the scale plus
    one rounding on each side); u' = fl(m u + gs) by that plus 2**-23 |u'|; v' = fl(v + u') by
    that plus 2**-23 |v'|.  Algorithm 4 adds gs twice and rounds four times after it
    (s = u + gs, u' = m s, w = v + u', v' = w + gs; |s| < 1.2 |u'| for m >= 0.85, |w| <=
    |v'| + |gs|)."""
    gs, u1, v1 = (np.abs(x).astype(np.float64) for x in (gs, u1, v1))
    if not nesterov:
        return 2.0 ** -22 * gs + 2.0 ** -23 * (u1 + v1)
    return 2.0 ** -21 * gs + 2.0 ** -23 * (2.2 * u1 + 2.0 * v1 + gs)


def flip_allowance(gs, u1, v1, thr, nesterov=False):
    """How far from the threshold an element may lie and still land on the other side of it
    when the clipping scale differs in its last bit: the element's own reach, the reach of the
    threshold (itself the v' of a sampled element; |gs|, |u'| <= |v'| = thr assumed there) and
    one unit in the last place of the threshold, which is the clause the comparison bar states."""
    thr = max(float(thr), 0.0)
    own = scale_reach(gs, u1, v1, nesterov)
    of_thr = float(scale_reach(np.float64(thr), np.float64(thr), np.float64(thr), nesterov))
    return own + of_thr + np.float64(np.spacing(np.float32(thr)))


def check_own_scale_run(pair, g, u0, v0, res, own, label):
    """The library's run on its own clipping scale against the oracle's result `res`
    (which used the oracle's scale), both from state (u0, v0)."""
    diag, per_idx, per_val, counts, thr = own
    assert abs(diag.norm - res.norm) <= 1e-6 * res.norm, (label, "norm", diag.norm, res.norm)
    assert abs(float(diag.scale) - float(res.scale)) <= 1e-6 * float(res.scale), (label, "scale")
    if np.float32(diag.scale) == res.scale:
        assert np.array_equal(thr.view(np.uint32), res.thresholds.view(np.uint32)), (label, "own-scale thresholds")
        if pair.sorted or not res.overflow:
            for j in range(pair.T):
                assert np.array_equal(per_idx[j], res.indices[j]), (label, "own-scale index set", j)
                assert np.array_equal(per_val[j].view(np.uint32), res.values[j].view(np.uint32)), (label, "own", j)
        return 0
    say(f"[parity] {label}: the library's clip scale differs from the oracle's in the last bit; tolerance rule")
    return compare_under_scale_tolerance(pair, g, u0, v0, res, per_idx, per_val, thr, pair.u.cpu().numpy(),
                                         pair.v.cpu().numpy(), label)


def compare_under_scale_tolerance(pair, g, u0, v0, res, per_idx, per_val, thr, u_dev, v_dev, label):
    """Comparison bar for a library run whose binary32 scale is not the oracle's: thresholds and
    sent values within 1e-6 relative; index sets differing only near the threshold; u and v
    within the reach of a last-bit change of the scale.  Returns the number of index flips."""
    ocfg = pair.ocfg
    u1, v1 = O.momentum_correction(g, u0, v0, ocfg.momentum, res.scale, ocfg.nesterov)
    gs = g * np.float32(res.scale)
    flips = 0
    worst_ulps = 0.0
    for j in range(pair.T):
        t_o = float(res.thresholds[j])
        assert abs(float(thr[j]) - t_o) <= 1e-6 * abs(t_o), (label, "threshold", j, thr[j], t_o)
        if res.overflow and not pair.sorted:
            continue
        a, b = per_idx[j].astype(np.int64), res.indices[j].astype(np.int64)
        common, ia, ib = np.intersect1d(a, b, assume_unique=True, return_indices=True)
        va, vb = per_val[j][ia].astype(np.float64), res.values[j][ib].astype(np.float64)
        assert np.all(np.abs(va - vb) <= 1e-6 * np.abs(vb)), (label, "values", j)
        diff = np.setxor1d(a, b, assume_unique=True)
        if diff.size:
            dist = np.abs(np.abs(v1[diff]).astype(np.float64) - t_o)
            allow = flip_allowance(gs[diff], u1[diff], v1[diff], t_o, ocfg.nesterov)
            assert np.all(dist <= allow), (label, "index flip away from the threshold", j, diff[:5], dist[:5], allow[:5])
            flips += int(diff.size)
            worst_ulps = max(worst_ulps, float((dist / np.spacing(np.float32(t_o))).max()))
    # state: unsent elements carry u', v' moved by the scale; sent ones are zero on both sides
    sent = np.zeros(pair.n, bool)
    for j in range(pair.T):
        sent[per_idx[j]] = True
        sent[res.indices[j]] = True
    reach = scale_reach(gs, u1, v1, ocfg.nesterov)
    keep = ~sent
    assert np.all(np.abs(v_dev.astype(np.float64) - pair.ov)[keep] <= reach[keep]), (label, "v under tolerance")
    assert np.all(np.abs(u_dev.astype(np.float64) - pair.ou)[keep] <= reach[keep]), (label, "u under tolerance")
    say(f"[parity] {label}: {flips} index flips, farthest {worst_ulps:.2f} ulp of the threshold from it")
    return flips


class Pair:
    """One worker on both sides."""

    def __init__(self, offsets, layout_density=None, capacities=None, warmup_workspace=False, **cfg_kw):
        import torch
        self.torch = torch
        self.offsets = [int(x) for x in offsets]
        self.n = self.offsets[-1]
        self.T = len(self.offsets) - 1
        self.cfg_kw = dict(cfg_kw)
        self.ocfg = oracle_config(**cfg_kw)
        self.sorted = bool(cfg_kw.get("flags", 0) & B.DGC_FLAG_SORTED_OUTPUT)
        self.dgc = B.Dgc(B.make_config(**cfg_kw), self.offsets, warmup_workspace=warmup_workspace)
        if capacities is not None:
            layout = np.concatenate([[0], np.cumsum(capacities)]).tolist()
        else:
            layout = self.dgc.dgc_recommended_payload_layout(
                layout_density if layout_density is not None else self.ocfg.density)
        # the oracle always sees the capacities the library was given
        self.capacities = [int(layout[j + 1] - layout[j]) for j in range(self.T)]
        self.dgc.set_layout(layout)
        self.layout = layout
        dev = "cuda"
        self.u = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.v = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.out_idx, self.out_val, self.out_counts, self.out_thr = self.dgc.alloc_payload(dev)
        self.ou = np.zeros(self.n, np.float32)
        self.ov = np.zeros(self.n, np.float32)
        self.last = None

    def set_density(self, d: float) -> None:
        self.dgc.dgc_set_density(d)
        self.ocfg.density = d

    def set_state(self, u: np.ndarray, v: np.ndarray) -> None:
        self.u.copy_(self.torch.from_numpy(u))
        self.v.copy_(self.torch.from_numpy(v))
        self.ou[:] = u
        self.ov[:] = v

    def run_library(self, g_dev, iteration):
        self.dgc.dgc_compress(g_dev, self.u, self.v, self.out_idx, self.out_val, self.out_counts,
                              self.out_thr, iteration)
        diag = self.dgc.dgc_get_diagnostics()
        per_idx, per_val, counts = gather_payload(self.layout, self.out_idx, self.out_val, self.out_counts,
                                                  sort=not self.sorted)
        return diag, per_idx, per_val, counts, self.out_thr.cpu().numpy()

    def step(self, g: np.ndarray, iteration: int, check_state: bool = True, label: str = ""):
        torch = self.torch
        g_dev = torch.from_numpy(g).cuda()
        u0, v0 = self.ou.copy(), self.ov.copy()
        res = O.compress(g, self.ou, self.ov, self.offsets, self.ocfg, iteration, self.capacities)
        clip = self.ocfg.clip_threshold > 0 and self.ocfg.scale_override is None
        if clip:
            # (own) the library's own clipping scale, from a copy of the device state
            u_keep, v_keep = self.u.clone(), self.v.clone()
            own = self.run_library(g_dev, iteration)
            check_own_scale_run(self, g, u0, v0, res, own, label)
            self.u.copy_(u_keep)
            self.v.copy_(v_keep)
            del u_keep, v_keep
            # (injected) the oracle's scale handed to the library
            self.dgc.dgc_set_scale_override(float(res.scale))
            diag, per_idx, per_val, counts, thr = self.run_library(g_dev, iteration)
            self.dgc.dgc_set_scale_override(float("nan"))
            assert abs(diag.norm - res.norm) <= 1e-6 * res.norm, (label, diag.norm, res.norm)
        else:
            diag, per_idx, per_val, counts, thr = self.run_library(g_dev, iteration)
        assert np.float32(diag.scale) == res.scale, (label, diag.scale, res.scale)

        assert np.array_equal(thr.view(np.uint32), res.thresholds.view(np.uint32)), \
            (label, "thresholds", np.flatnonzero(thr != res.thresholds)[:5])
        assert np.array_equal(counts.astype(np.int64), res.counts), (label, "counts")
        overflow = bool(diag.flags & B.DGC_DIAG_OVERFLOW)
        assert overflow == res.overflow, (label, "overflow flag")
        if self.sorted or not res.overflow:
            for j in range(self.T):
                assert np.array_equal(per_idx[j], res.indices[j]), (label, "index set", j)
                assert np.array_equal(per_val[j].view(np.uint32), res.values[j].view(np.uint32)), \
                    (label, "values", j)
            if check_state:
                assert np.array_equal(self.u.cpu().numpy().view(np.uint32), self.ou.view(np.uint32)), (label, "u")
                assert np.array_equal(self.v.cpu().numpy().view(np.uint32), self.ov.view(np.uint32)), (label, "v")
        self.last = (res, per_idx, per_val, counts, diag)
        return res

    def device_payload(self):
        return self.out_idx, self.out_val, self.out_counts

    def close(self):
        self.dgc.close()


def check_overflow_invariants(pair: Pair, g: np.ndarray, u0: np.ndarray, v0: np.ndarray):
    """Under capacity overflow which elements are dropped is order-dependent; what must
    hold is conservation, the mask rule, and full regions."""
    res, per_idx, per_val, counts, diag = pair.last
    u_dev = pair.u.cpu().numpy()
    v_dev = pair.v.cpu().numpy()
    u1, v1 = O.momentum_correction(g, u0, v0, pair.ocfg.momentum, res.scale, pair.ocfg.nesterov)
    sent = np.zeros(pair.n, np.float32)
    mask = np.zeros(pair.n, bool)
    for j in range(pair.T):
        cap = pair.layout[j + 1] - pair.layout[j]
        assert per_idx[j].size == min(int(counts[j]), cap)
        assert np.unique(per_idx[j]).size == per_idx[j].size
        lo, hi = pair.offsets[j], pair.offsets[j + 1]
        assert np.all((per_idx[j] >= lo) & (per_idx[j] < hi))
        assert np.all(np.abs(v1[per_idx[j]]) > res.thresholds[j])
        sent[per_idx[j]] = per_val[j]
        mask[per_idx[j]] = True
    assert np.array_equal(np.where(mask, sent, v_dev).view(np.uint32), v1.view(np.uint32))
    u_expect = np.where(mask, np.float32(0), u1) if pair.ocfg.factor_masking else u1
    assert np.array_equal(u_dev.view(np.uint32), u_expect.view(np.uint32))
    assert np.all(v_dev[mask] == 0)
