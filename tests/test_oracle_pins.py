"""Pins for the CPU oracle: each test checks it against something the paper or
the mathematics fixes, computed here by other means (pure-Python loops, closed
forms, textbook recurrences), never by calling the oracle's own formula again.
"""

import math
import os

import numpy as np
import pytest

from oracle import dgc_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
f32 = np.float32


def cfg(**kw):
    base = dict(momentum=0.9, density=0.25, sample_min=8, sample_max=64, sample_block=4,
                sample_ratio=0.01, seed=3)
    base.update(kw)
    return O.OracleConfig(**base)


# ---------------------------------------------------------------------------
# P1  brute-force top-k on tiny tensors (Algorithm 3: threshold + strict mask)
# ---------------------------------------------------------------------------
def brute_topk_strict(values, k):
    """Indices sent when the threshold is the (k+1)-th largest magnitude and the
    comparison is strict; everything when k >= len."""
    mags = [abs(float(x)) for x in values]
    if k >= len(mags):
        return list(range(len(mags)))
    order = sorted(mags, reverse=True)
    thr = order[k]
    return [i for i, a in enumerate(mags) if a > thr]


@pytest.mark.parametrize("vals,density", [
    ([0.5, -3.0, 2.0, 0.1, -0.2, 1.0, 7.0, -6.0], 0.25),      # k = 2: sends 7, -6
    ([0.5, -3.0, 2.0, 0.1, -0.2, 1.0, 7.0, -6.0], 0.125),     # k = 1
    ([0.5, -3.0, 2.0, 0.1, -0.2, 1.0, 7.0, -6.0], 1.0),       # k = n: everything
    ([1.0, 1.0, 1.0, 1.0], 0.5),                              # all tied: nothing passes strict >
    ([0.0, 0.0, 5.0, 0.0, 0.0, 0.0, 0.0, 0.0], 0.5),          # fewer non-zeros than k: thr = 0
    ([2.0, -2.0, 1.0, 3.0], 0.5),                             # tie at the boundary
    ([-0.0, 0.0, 1e-45, -1e-45], 0.25),                       # signed zeros and denormals
])
def test_p1_exact_topk_matches_bruteforce(vals, density):
    g = np.array(vals, dtype=f32)
    n = g.size
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    c = cfg(momentum=0.0, density=density, exact_select=True)
    res = O.compress(g, u, v, [0, n], c, 0)
    k = max(1, min(n, math.ceil(density * n)))
    expect = brute_topk_strict(vals, k)
    assert res.indices[0].tolist() == expect
    assert [float(x) for x in res.values[0]] == [float(f32(vals[i])) for i in expect]
    assert int(res.counts[0]) == len(expect)


def test_p1_hand_example():
    # eight elements, density 0.25 -> k = 2; magnitudes sorted: 7 6 3 2 1 .5 .2 .1;
    # threshold = third largest = 3; sent = {7, -6}.
    g = np.array([0.5, -3.0, 2.0, 0.1, -0.2, 1.0, 7.0, -6.0], dtype=f32)
    u = np.zeros(8, f32)
    v = np.zeros(8, f32)
    res = O.compress(g, u, v, [0, 8], cfg(momentum=0.0, density=0.25, exact_select=True), 0)
    assert float(res.thresholds[0]) == 3.0
    assert res.indices[0].tolist() == [6, 7]
    assert res.values[0].tolist() == [7.0, -6.0]
    assert v.tolist() == [0.5, -3.0, 2.0, 0.1 + 0.0, -0.2 + 0.0, 1.0, 0.0, 0.0] or \
        np.array_equal(v, np.array([0.5, -3.0, 2.0, 0.1, -0.2, 1.0, 0.0, 0.0], f32))


def test_p1_random_small_against_bruteforce():
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(1, 65))
        d = float(rng.choice([0.01, 0.1, 0.3, 0.5, 0.99, 1.0]))
        vals = rng.integers(-6, 7, size=n).astype(f32) * f32(0.25)   # many ties and zeros
        u = np.zeros(n, f32)
        v = np.zeros(n, f32)
        res = O.compress(vals.copy(), u, v, [0, n], cfg(momentum=0.0, density=d, exact_select=True), trial)
        k = max(1, min(n, math.ceil(d * n)))
        assert res.indices[0].tolist() == brute_topk_strict(vals.tolist(), k)


# ---------------------------------------------------------------------------
# P4  exact mode sends ceil(d n) when magnitudes are distinct
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,d", [(1000, 0.001), (1000, 0.0015), (4097, 0.001), (1 << 20, 0.001),
                                 (64, 0.001), (777, 0.25), (10, 1.0)])
def test_p4_count_is_ceil_dn(n, d):
    rng = np.random.default_rng(n)
    g = (rng.permutation(n).astype(np.float64) + 1.0).astype(f32)   # distinct magnitudes
    g *= rng.choice([-1.0, 1.0], size=n).astype(f32)
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    res = O.compress(g, u, v, [0, n], cfg(momentum=0.0, density=d, exact_select=True), 0)
    assert int(res.counts[0]) == max(1, min(n, math.ceil(d * n)))
    if n == 1 << 20:
        assert int(res.counts[0]) == 1049       # the toy configuration's k


def test_topk_count_clamps():
    assert O.topk_count(0.001, 64) == 1
    assert O.topk_count(1.0, 64) == 64
    assert O.topk_count(0.001, 1048576) == 1049
    assert O.topk_count(0.001, 2359296) == 2360


# ---------------------------------------------------------------------------
# P2  conservation and momentum factor masking (Algorithm 3, mask lines)
# ---------------------------------------------------------------------------
def python_update(g, u, v, m, scale, nesterov=False):
    """Scalar loop over binary32 values, one rounding per operation."""
    u1 = np.empty_like(u)
    v1 = np.empty_like(v)
    m = f32(m)
    scale = f32(scale)
    for i in range(g.size):
        gs = f32(g[i] * scale)
        if not nesterov:
            t = f32(m * u[i])
            u1[i] = f32(t + gs)
            v1[i] = f32(v[i] + u1[i])
        else:
            s = f32(u[i] + gs)
            u1[i] = f32(m * s)
            w = f32(v[i] + u1[i])
            v1[i] = f32(w + gs)
    return u1, v1


@pytest.mark.parametrize("nesterov", [False, True])
@pytest.mark.parametrize("factor_masking", [True, False])
def test_p2_conservation_and_masks(nesterov, factor_masking):
    rng = np.random.default_rng(11)
    offsets = [0, 37, 38, 300, 1324]
    n = offsets[-1]
    u = (rng.standard_normal(n) * 0.1).astype(f32)
    v = (rng.standard_normal(n) * 0.1).astype(f32)
    c = cfg(density=0.05, nesterov=nesterov, factor_masking=factor_masking)
    for it in range(3):
        g = rng.standard_t(3, n).astype(f32)
        u1, v1 = python_update(g, u, v, 0.9, 1.0, nesterov)
        res = O.compress(g, u, v, offsets, c, it)
        idx, val = O.flatten_payload(res)
        sent = np.zeros(n, f32)
        sent[idx] = val
        mask = np.zeros(n, bool)
        mask[idx] = True
        # every pre-mask value is either in the payload or left in v, bit for bit
        assert np.array_equal(np.where(mask, sent, v).view(np.uint32), v1.view(np.uint32))
        assert np.all(v[mask] == 0.0)
        # u is cleared exactly where v is (or nowhere when factor masking is off)
        expect_u = np.where(mask, f32(0), u1) if factor_masking else u1
        assert np.array_equal(u.view(np.uint32), expect_u.view(np.uint32))
        # the mask is the strict comparison with the per-tensor threshold
        for j in range(len(offsets) - 1):
            lo, hi = offsets[j], offsets[j + 1]
            assert np.array_equal(mask[lo:hi], np.abs(v1[lo:hi]) > res.thresholds[j])


def test_p2_capacity_overflow_keeps_conservation():
    rng = np.random.default_rng(12)
    n = 512
    g = rng.standard_normal(n).astype(f32)
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    res = O.compress(g, u, v, [0, n], cfg(momentum=0.0, density=0.25, exact_select=True), 0,
                     capacities=[10])
    assert res.overflow and int(res.counts[0]) == 128 and res.indices[0].size == 10
    sent = np.zeros(n, f32)
    sent[res.indices[0]] = res.values[0]
    assert np.array_equal(sent + v, g)
    assert np.count_nonzero(sent) == 10


# ---------------------------------------------------------------------------
# P3  density 1: dense momentum SGD (Eq. 3) / plain SGD
# ---------------------------------------------------------------------------
def test_p3a_density_one_no_factor_masking_is_momentum_sgd():
    rng = np.random.default_rng(21)
    n = 257
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    vel = np.zeros(n, f32)       # textbook velocity: u_t = m u_{t-1} + grad_t  (Eq. 3, one node)
    c = cfg(density=1.0, factor_masking=False)
    for it in range(6):
        g = rng.standard_normal(n).astype(f32)
        for i in range(n):
            vel[i] = f32(f32(f32(0.9) * vel[i]) + g[i])
        res = O.compress(g, u, v, [0, 100, n], c, it)
        idx, val = O.flatten_payload(res)
        assert idx.tolist() == list(range(n))
        assert np.array_equal(val.view(np.uint32), vel.view(np.uint32))
        assert not v.any()


def test_p3b_density_one_with_factor_masking_is_sgd():
    rng = np.random.default_rng(22)
    n = 100
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    for it in range(4):
        g = rng.standard_normal(n).astype(f32)
        res = O.compress(g, u, v, [0, n], cfg(density=1.0), it)
        idx, val = O.flatten_payload(res)
        assert np.array_equal(val, g) and idx.size == n
        assert not u.any() and not v.any()


def test_p3c_nesterov_density_one_matches_eq8():
    # Nesterov SGD (Appendix B, first equation): u_{t+1} = m u_t + grad; step = m u_{t+1} + grad.
    # With factor masking off and density 1 the payload of Algorithm 4 is that step,
    # and Algorithm 4's U equals m times the equation's u.
    rng = np.random.default_rng(23)
    n = 64
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    ueq = np.zeros(n, np.float64)
    for it in range(5):
        g = rng.standard_normal(n).astype(f32)
        ueq = 0.9 * ueq + g.astype(np.float64)
        step = 0.9 * ueq + g
        res = O.compress(g, u, v, [0, n], cfg(density=1.0, nesterov=True, factor_masking=False), it)
        _, val = O.flatten_payload(res)
        np.testing.assert_allclose(val, step, rtol=2e-6, atol=2e-6)   # values reach ~10
        np.testing.assert_allclose(u, 0.9 * ueq, rtol=2e-6, atol=2e-6)


# ---------------------------------------------------------------------------
# P5  accumulated discount factor of an unsent coordinate (Eq. 4 / Eq. 7)
# ---------------------------------------------------------------------------
def test_p5_geometric_discount_factor():
    n = 16
    m = 0.9
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    c = cfg(momentum=m, density=1.0 / 16, exact_select=True)
    T = 12
    for t in range(T):
        g = np.zeros(n, f32)
        g[0] = 1000.0          # a large decoy that is sent every iteration
        if t == 0:
            g[5] = 1.0         # impulse on an unsent coordinate
        g[7] = 0.5             # constant gradient on another unsent coordinate
        res = O.compress(g, u, v, [0, n], c, t)
        assert res.indices[0].tolist() == [0]
        tt = t + 1
        impulse = (1.0 - m ** tt) / (1.0 - m)
        const = 0.5 * sum((1.0 - m ** s) / (1.0 - m) for s in range(1, tt + 1))
        assert abs(float(v[5]) - impulse) <= 4e-6 * impulse
        assert abs(float(v[7]) - const) <= 4e-6 * const


# ---------------------------------------------------------------------------
# P6  m = 0 is Algorithm 1 (plain local accumulation)
# ---------------------------------------------------------------------------
def test_p6_zero_momentum_is_running_sum():
    rng = np.random.default_rng(31)
    n = 400
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    acc = np.zeros(n, f32)
    for it in range(5):
        g = rng.standard_normal(n).astype(f32)
        acc = acc + g                                  # Algorithm 1: G_t <- G_{t-1} + grad
        k = math.ceil(0.05 * n)
        thr = np.sort(np.abs(acc))[::-1][k]
        mask = np.abs(acc) > thr
        res = O.compress(g, u, v, [0, n], cfg(momentum=0.0, density=0.05, exact_select=True), it)
        assert res.indices[0].tolist() == np.flatnonzero(mask).tolist()
        assert np.array_equal(res.values[0], acc[mask])
        acc[mask] = 0
        assert np.array_equal(v, acc)


# ---------------------------------------------------------------------------
# P7  local gradient clipping (Appendix C, Eq. 12)
# ---------------------------------------------------------------------------
def test_p7_clip_scale():
    rng = np.random.default_rng(41)
    g = rng.standard_normal(10000).astype(f32)           # norm ~ 100
    norm, scale = O.clip_scale(g, 1.0, 4)
    brute = math.sqrt(math.fsum(float(x) * float(x) for x in g))
    assert abs(norm - brute) <= 1e-12 * brute
    clipped = g.astype(np.float64) * float(scale)
    assert abs(np.linalg.norm(clipped) - 0.5) <= 1e-6 * 0.5   # thr_G / sqrt(N) = 1/2
    # below the local threshold nothing is rescaled
    small = (g * f32(1e-4)).astype(f32)
    _, s2 = O.clip_scale(small, 1.0, 4)
    assert s2 == f32(1.0)
    # N enters as N**-0.5
    _, s16 = O.clip_scale(g, 1.0, 16)
    assert abs(float(s16) / float(scale) - 0.5) < 1e-6


def test_p7_clipping_is_applied_before_accumulation():
    rng = np.random.default_rng(42)
    n = 300
    g = rng.standard_normal(n).astype(f32)
    u = np.full(n, 0.25, f32)
    v = np.full(n, -0.5, f32)
    u0, v0 = u.copy(), v.copy()
    c = cfg(density=1e-9, clip_threshold=2.0, num_workers=4, exact_select=True)
    res = O.compress(g, u, v, [0, n], c, 0)
    assert res.scale < 1.0
    u1, v1 = python_update(g, u0, v0, 0.9, res.scale)
    sent = int(res.indices[0][0])
    keep = np.ones(n, bool)
    keep[sent] = False
    assert np.array_equal(u[keep], u1[keep]) and np.array_equal(v[keep], v1[keep])


# ---------------------------------------------------------------------------
# P8  a sample that is the whole tensor is exact mode; refinement gives exact top-k
# ---------------------------------------------------------------------------
def test_p8_small_tensor_sampled_equals_exact():
    rng = np.random.default_rng(51)
    n = 50                                   # below sample_min -> identity sample
    g = rng.standard_normal(n).astype(f32)
    a = O.compress(g, np.zeros(n, f32), np.zeros(n, f32), [0, n], cfg(sample_min=64), 0)
    b = O.compress(g, np.zeros(n, f32), np.zeros(n, f32), [0, n], cfg(sample_min=64, exact_select=True), 0)
    assert a.indices[0].tolist() == b.indices[0].tolist() and a.thresholds[0] == b.thresholds[0]


def test_p8_refinement_yields_exact_topk():
    rng = np.random.default_rng(52)
    n = 20000
    c_s = cfg(density=0.01, sample_min=64, sample_max=64, sample_block=4, refine_alpha=1.0)
    c_e = cfg(density=0.01, exact_select=True)
    hit = 0
    for it in range(20):
        g = rng.standard_t(3, n).astype(f32)
        a = O.compress(g, np.zeros(n, f32), np.zeros(n, f32), [0, n], c_s, it)
        if a.refined[0]:
            hit += 1
            b = O.compress(g, np.zeros(n, f32), np.zeros(n, f32), [0, n], c_e, it)
            assert a.indices[0].tolist() == b.indices[0].tolist()
            assert int(a.counts[0]) == 200
    assert hit >= 3


# ---------------------------------------------------------------------------
# Sampled threshold: rank rule on the sample (Section 5)
# ---------------------------------------------------------------------------
def test_sampled_threshold_estimates_population_quantile():
    rng = np.random.default_rng(61)
    n = 1 << 20
    c = O.OracleConfig(momentum=0.0, density=0.001, seed=9)
    plan = O.sample_plan(n, c)
    # the toy configuration's plan: 1 % of 2**20 in blocks of 32, rank ceil(0.001 * 10496)
    assert (plan.exact, plan.blocks, plan.count, plan.rank, plan.k) == (False, 328, 10496, 11, 1049)
    counts = []
    for it in range(12):
        g = (1e-3 * rng.standard_t(3, n)).astype(f32)
        res = O.compress(g, np.zeros(n, f32), np.zeros(n, f32), [0, n], c, it)
        counts.append(int(res.counts[0]))
        assert int(res.counts[0]) == int(np.count_nonzero(np.abs(g) > res.thresholds[0]))
    mean = float(np.mean(counts))
    # an order statistic of rank 11 in a sample: relative spread ~ 1/sqrt(11); mean within 25 %
    assert 0.75 * 1049 < mean < 1.25 * 1049
    assert min(counts) > 300 and max(counts) < 3000


def test_sample_plan_rules():
    c = O.OracleConfig(density=0.001)
    p = O.sample_plan(4096, c)
    assert p.exact and p.count == 4096 and p.rank == 5
    p = O.sample_plan(4097, c)
    assert (not p.exact) and p.blocks == 128 and p.count == 4096 and p.rank == 5 and p.nblocks == 128
    p = O.sample_plan(2359296, c)              # ResNet-50's largest tensor: 1 % = 23593
    assert p.blocks == 738 and p.count == 23616 and p.rank == 24 and p.k == 2360
    p = O.sample_plan(15000000, c)             # capped at sample_max
    assert p.count == 32768 and p.rank == 33
    p = O.sample_plan(4723200, c, density=0.25)
    assert p.count == 32768 and p.rank == 8192 and p.k == 1180800


# ---------------------------------------------------------------------------
# P11  sample positions
# ---------------------------------------------------------------------------
def test_p11_sample_positions_properties():
    c = O.OracleConfig(density=0.001, seed=1234)
    n = 100003
    plan = O.sample_plan(n, c)
    pos = O.sample_positions(c.seed, 7, 3, plan, c.sample_block)
    B = c.sample_block
    assert pos.size == plan.count and pos.min() >= 0 and pos.max() < (n // B) * B
    blocks = pos.reshape(-1, B)
    assert np.all(blocks[:, 0] % B == 0)
    assert np.all(np.diff(blocks, axis=1) == 1)
    assert np.array_equal(pos, O.sample_positions(c.seed, 7, 3, plan, c.sample_block))
    for other in [(c.seed + 1, 7, 3), (c.seed, 8, 3), (c.seed, 7, 4), (c.seed + (1 << 32), 7, 3),
                  (c.seed, 7 + (1 << 32), 3)]:
        assert not np.array_equal(pos, O.sample_positions(*other, plan, c.sample_block))


def test_p11_mixer_is_a_bijection_on_a_slice_and_uniform():
    x = np.arange(1 << 20, dtype=np.uint64)
    y = O.mix32(x)
    assert np.unique(y).size == x.size and y.max() <= 0xFFFFFFFF
    # block ids drawn for a long stream are uniform: chi-square over 64 cells
    plan = O.SamplePlan(False, 16 * 200000, 1, 200000, 64, 1)
    pos = O.sample_positions(1, 2, 3, plan, 16)
    cells = np.bincount((pos[::16] // 16).astype(np.int64), minlength=64)
    chi2 = float(np.sum((cells - 200000 / 64) ** 2 / (200000 / 64)))
    assert chi2 < 120.0        # 63 degrees of freedom: 99.99 % quantile ~ 113


# ---------------------------------------------------------------------------
# P9  telescoping: everything is eventually sent (Section 3.1)
# ---------------------------------------------------------------------------
def test_p9_sent_plus_residual_equals_dense_velocity_sum():
    rng = np.random.default_rng(71)
    n = 2000
    u = np.zeros(n, f32)
    v = np.zeros(n, f32)
    vel = np.zeros(n, np.float64)
    vel_sum = np.zeros(n, np.float64)
    sent_sum = np.zeros(n, np.float64)
    c = cfg(density=0.02, factor_masking=False)
    for it in range(30):
        g = rng.standard_normal(n).astype(f32)
        vel = 0.9 * vel + g
        vel_sum += vel
        res = O.compress(g, u, v, [0, 700, n], c, it)
        idx, val = O.flatten_payload(res)
        sent_sum[idx] += val
    np.testing.assert_allclose(sent_sum + v, vel_sum, rtol=1e-5, atol=1e-5)


# ---------------------------------------------------------------------------
# P10  receive side is a dense sum (Algorithm 2's all-reduce line)
# ---------------------------------------------------------------------------
def test_p10_decompress_is_dense_sum():
    rng = np.random.default_rng(81)
    n = 5000
    N = 5
    dense_parts = []
    payloads = []
    for w in range(N):
        idx = np.sort(rng.choice(n, size=300, replace=False)).astype(np.int32)
        val = rng.standard_normal(300).astype(f32)
        d = np.zeros(n, f32)
        d[idx] = val
        dense_parts.append(d)
        payloads.append((idx, val))
    out = np.zeros(n, f32)
    O.decompress_accumulate(out, payloads)
    expect = np.zeros(n, f32)
    for d in dense_parts:                      # worker order, binary32
        expect = expect + d
    assert np.array_equal(out, expect)
    # accumulates into what is there, does not overwrite; no division by N
    O.decompress_accumulate(out, payloads[:1])
    assert np.array_equal(out, expect + dense_parts[0])


def test_p10_density_one_all_workers_equals_sum_of_v():
    rng = np.random.default_rng(82)
    n = 300
    N = 3
    total = np.zeros(n, f32)
    payloads = []
    for w in range(N):
        g = rng.standard_normal(n).astype(f32)
        res = O.compress(g, np.zeros(n, f32), np.zeros(n, f32), [0, n], cfg(density=1.0), 0)
        payloads.append(O.flatten_payload(res))
        total = total + g
    out = np.zeros(n, f32)
    O.decompress_accumulate(out, payloads)
    assert np.array_equal(out, total)


def test_sparse_sgd_apply_is_dense_sgd_on_the_aggregate():
    # theta - lr * G_t with G_t = sum of the workers' sparse gradients (Algorithm 3, last two lines)
    rng = np.random.default_rng(83)
    n, N, lr = 4000, 4, 0.05
    theta0 = rng.standard_normal(n).astype(f32)
    payloads = []
    G = np.zeros(n, np.float64)
    for w in range(N):
        idx = np.sort(rng.choice(n, size=500, replace=False)).astype(np.int32)
        val = rng.standard_normal(500).astype(f32)
        payloads.append((idx, val))
        G[idx] += val
    theta = theta0.copy()
    O.sparse_sgd_apply(theta, payloads, lr)
    np.testing.assert_allclose(theta, theta0 - lr * G, rtol=0, atol=4e-7 * (np.abs(theta0) + lr * 4 * 4).max())
    untouched = G == 0
    assert np.array_equal(theta[untouched], theta0[untouched])
    # an index that occurs once is updated with exactly two roundings
    once = np.zeros(n, int)
    for idx, _ in payloads:
        once[idx] += 1
    single = once == 1
    dense32 = np.zeros(n, f32)
    O.decompress_accumulate(dense32, payloads)
    expect = theta0 - f32(lr) * dense32
    assert np.array_equal(theta[single], expect[single])


# ---------------------------------------------------------------------------
# Wire format: 32-bit values + 16-bit zero-run lengths (Section 3.1)
# ---------------------------------------------------------------------------
def brute_decode(n, runs, vals):
    out = [0.0] * n
    pos = 0
    for r, x in zip(runs, vals):
        for _ in range(int(r)):
            pos += 1                       # a zero
        out[pos] = float(x)
        pos += 1
    return out


def test_encode_hand_example():
    # dense vector 0 0 5 0 0 0 -2 7 0 -> runs 2, 3, 0 and values 5, -2, 7 (trailing zero not sent)
    runs, vals = O.encode(np.array([7, 2, 6]), np.array([7.0, 5.0, -2.0], f32))
    assert runs.tolist() == [2, 3, 0] and vals.tolist() == [5.0, -2.0, 7.0]
    assert runs.dtype == np.uint16 and vals.dtype == f32
    assert O.encoded_bytes(len(runs)) == 18
    assert brute_decode(9, runs, vals) == [0, 0, 5, 0, 0, 0, -2, 7, 0]


def test_encode_long_runs_use_filler_entries():
    # first value after exactly 65535 zeros fits one entry; after 65536 it needs a filler
    r, v = O.encode(np.array([65535]), np.array([1.0], f32))
    assert r.tolist() == [65535] and v.tolist() == [1.0]
    r, v = O.encode(np.array([65536]), np.array([1.0], f32))
    assert r.tolist() == [65535, 0] and v.tolist() == [0.0, 1.0]
    r, v = O.encode(np.array([3, 3 + 1 + 200000]), np.array([1.0, 2.0], f32))
    assert r.tolist() == [3, 65535, 65535, 65535, 200000 - 3 * 65536] and v.tolist() == [1.0, 0.0, 0.0, 0.0, 2.0]
    dense = np.zeros(200010, f32)
    O.decode_accumulate(dense, r, v)
    assert dense[3] == 1.0 and dense[200004] == 2.0 and np.count_nonzero(dense) == 2


def test_encode_decode_round_trip_random():
    rng = np.random.default_rng(91)
    for trial in range(30):
        n = int(rng.integers(1, 400000))
        k = int(rng.integers(0, min(n, 300) + 1))
        idx = rng.choice(n, size=k, replace=False)
        val = rng.standard_normal(k).astype(f32)
        runs, vals = O.encode(idx, val)
        expect = np.zeros(n, f32)
        expect[idx] = val
        if n <= 5000:
            assert brute_decode(n, runs, vals) == expect.tolist()
        got = np.ones(n, f32)
        O.decode_accumulate(got, runs, vals)
        assert np.array_equal(got, expect + f32(1.0))            # accumulates, does not overwrite
        fillers = int(np.count_nonzero((runs == 65535) & (vals == 0)))
        assert len(runs) <= k + n // 65536 and len(runs) >= k
        assert len(runs) - k <= fillers


# ---------------------------------------------------------------------------
# Values the paper prints
# ---------------------------------------------------------------------------
def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def test_warmup_schedule_matches_paper_sparsities():
    rows = _golden_rows("warmup_sparsity_percent.txt")
    printed = [float(r[0]) for r in rows]
    assert len(printed) == len(O.WARMUP_DENSITIES) == 5
    for p, d in zip(printed, O.WARMUP_DENSITIES):
        assert abs((1.0 - d) * 100.0 - p) < 0.011      # 99.6 is 99.609375 rounded
    assert O.warmup_density(O.WARMUP_DENSITIES, 0) == 0.25
    assert O.warmup_density(O.WARMUP_DENSITIES, 4) == 0.001
    assert O.warmup_density(O.WARMUP_DENSITIES, 400) == 0.001


def test_compression_ratio_accounting():
    # the tables print dense/payload; at 0.1 % with 6-byte entries that is 4/(6*0.001)
    assert abs(O.compression_ratio(1_000_000, 1000, 6) - 666.67) < 0.01
    assert abs(O.compression_ratio(1_000_000, 1000, 8) - 500.0) < 1e-9
