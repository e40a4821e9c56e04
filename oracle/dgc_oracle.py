"""CPU oracle for the per-worker hot path of Deep Gradient Compression.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
path computes, written from the paper (arXiv 1712.01887).  It is imported by the
tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
nothing else; the product (the HIP library and its Python binding) never calls
it, and it never imports the product.  It shares no code, table or constant
generator with the HIP path: the integer mixer that draws the sample positions
is implemented once here and once, independently, in the kernels.

What is taken from the paper and what is a reading of it:

* Algorithm 3 (Appendix D) gives the step order followed by `compress`:
  clip -> U <- m U + G -> V <- V + U -> per-tensor threshold -> mask ->
  sparse extract -> zero V and U under the mask.  Algorithm 4 gives the
  Nesterov form (`nesterov=True`).
* Equation 7 (Section 3.2) is the momentum-corrected accumulation.
* Appendix C, equation 12: the local clipping threshold is N**-0.5 times the
  global one; Section 3.2 places clipping before accumulation.
* Section 3.3 (unnumbered equation): the same mask clears V and U.
* Section 5: the threshold is estimated by a top-k selection on a sample of
  0.1 % to 1 % of the elements; if far too many elements pass, a precise
  threshold is recomputed from those already selected (`refine_alpha`).
* Algorithm 3's all-reduce line: the receive side is the plain sum of the
  N sparse gradients (`decompress_accumulate`).

The paper does not say how "s % of |V|" becomes a number, how the sample is
drawn, or in which precision anything runs.  The readings used here:
k = clamp(ceil(d*n), 1, n) evaluated in binary64; the threshold is the
magnitude of 0-based descending rank r in the candidate set (r = k in exact
mode, r = ceil(d*s') on a sample of s' elements) and -1 when r is not below
the set's size, so that the strict comparison of Algorithm 3 sends exactly k
elements when magnitudes are distinct; the elementwise work is binary32 with
every operation rounded on its own (no fused multiply-add), the clipping norm
is accumulated in binary64 and the scale is rounded once to binary32.

Parity pins: every function below is pinned by tests/test_oracle_pins.py
(brute-force top-k, conservation, dense limits, closed-form geometric sums,
the clipped norm, sample = whole tensor, statistical accuracy of the sampled
threshold, dense-sum equivalence of the receive side).  The sample-position
mixer has no value fixed by the paper; it is pinned by its properties only
(range, block alignment, reproducibility, bijectivity of the 32-bit mixer,
uniformity) -- parity unpinned for the constants themselves, which are a
free choice.  No compression ratio printed in the paper can be reproduced
without the trained gradients: parity unpinned for Tables 3 and 4.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_M32 = 0xFFFFFFFF


# --------------------------------------------------------------------------
# Configuration (mirrors the arguments of the method, Algorithm 3 "Require")
# --------------------------------------------------------------------------
@dataclass
class OracleConfig:
    momentum: float = 0.9            # m
    clip_threshold: float = 0.0      # thr_G of Appendix C; <= 0 turns clipping off
    num_workers: int = 1             # N
    density: float = 0.001           # d = 1 - sparsity
    sample_ratio: float = 0.01       # Section 5: 0.1 % .. 1 %
    sample_min: int = 4096
    sample_max: int = 32768
    sample_block: int = 32           # consecutive elements per draw (one 128-byte line)
    seed: int = 0
    nesterov: bool = False           # Algorithm 4 instead of Algorithm 3
    factor_masking: bool = True      # Section 3.3; False = ablation / Eq. 3 limit
    exact_select: bool = False       # threshold from the whole tensor
    scale_override: Optional[float] = None   # test hook: bypass the norm
    refine_alpha: Optional[float] = None     # Section 5 re-threshold; None = off


WARMUP_DENSITIES = (0.25, 0.0625, 0.015625, 0.004, 0.001)
"""Section 4.1: sparsity 75 %, 93.75 %, 98.4375 %, 99.6 %, 99.9 % as densities."""


def warmup_density(schedule: Sequence[float], iteration: int, stage_length: int = 1) -> float:
    """Density for an iteration: every schedule entry is held for `stage_length`
    iterations (an epoch in the paper's runs), the last one for good."""
    return float(schedule[min(int(iteration) // int(stage_length), len(schedule) - 1)])


# --------------------------------------------------------------------------
# Local gradient clipping (Section 3.2; Appendix C, equation 12)
# --------------------------------------------------------------------------
def clip_scale(g: np.ndarray, clip_threshold: float, num_workers: int
               ) -> Tuple[float, np.float32]:
    """Return (L2 norm of the whole gradient set, scale applied to it).

    The norm runs over every tensor of the worker's gradient, accumulated in
    binary64.  The local threshold is thr_G / sqrt(N).  The gradient is
    rescaled only when its norm exceeds the local threshold.
    """
    g64 = g.astype(np.float64)
    total = float(np.sum(g64 * g64))
    norm = math.sqrt(total)
    thr_local = float(np.float32(clip_threshold)) / math.sqrt(float(num_workers))
    if norm > thr_local:
        return norm, np.float32(thr_local / norm)
    return norm, np.float32(1.0)


# --------------------------------------------------------------------------
# Momentum correction (equation 7; Algorithm 3 / Algorithm 4 update lines)
# --------------------------------------------------------------------------
def momentum_correction(g: np.ndarray, u: np.ndarray, v: np.ndarray, m: float,
                        scale: np.float32, nesterov: bool = False
                        ) -> Tuple[np.ndarray, np.ndarray]:
    """Pre-mask velocity U_t and accumulation V_t, binary32, one rounding per op."""
    assert g.dtype == np.float32 and u.dtype == np.float32 and v.dtype == np.float32
    m32 = np.float32(m)
    gs = g * np.float32(scale)
    if not nesterov:
        t = m32 * u
        u1 = t + gs          # U <- m U + G
        v1 = v + u1          # V <- V + U
    else:
        s = u + gs
        u1 = m32 * s         # U <- m (U + G)
        w = v + u1
        v1 = w + gs          # V <- V + U + G
    return u1, v1


# --------------------------------------------------------------------------
# How many to send, how many to sample
# --------------------------------------------------------------------------
def topk_count(density: float, n: int) -> int:
    """k = ceil(d n) clamped to [1, n], product formed in binary64."""
    k = int(math.ceil(float(density) * float(n)))
    return max(1, min(int(n), k))


@dataclass
class SamplePlan:
    exact: bool      # candidates are the whole tensor
    count: int       # number of candidates (n, or blocks*block for a sample)
    rank: int        # 0-based descending rank whose magnitude is the threshold
    blocks: int      # draws (sampled mode)
    nblocks: int     # aligned blocks the tensor holds (sampled mode)
    k: int           # ceil(d n) for the whole tensor


def sample_plan(n: int, cfg: OracleConfig, density: Optional[float] = None) -> SamplePlan:
    d = cfg.density if density is None else density
    k = topk_count(d, n)
    want = int(math.ceil(float(cfg.sample_ratio) * float(n)))
    want = max(int(cfg.sample_min), min(int(cfg.sample_max), want))
    s = min(int(n), want)
    B = int(cfg.sample_block)
    if cfg.exact_select or s >= n or n // B < 1:
        return SamplePlan(True, int(n), k, 0, 0, k)
    blocks = (s + B - 1) // B
    count = blocks * B
    rank = max(1, int(math.ceil(float(d) * float(count))))
    return SamplePlan(False, count, rank, blocks, n // B, k)


# --------------------------------------------------------------------------
# Counter-based sample positions (a reading: the paper only says "sample")
# --------------------------------------------------------------------------
def mix32(x: np.ndarray) -> np.ndarray:
    """A 32-bit xorshift-multiply finaliser (a bijection on 32-bit words)."""
    x = np.asarray(x, dtype=np.uint64) & _M32
    x = x ^ (x >> np.uint64(16))
    x = (x * np.uint64(0x7FEB352D)) & _M32
    x = x ^ (x >> np.uint64(15))
    x = (x * np.uint64(0x846CA68B)) & _M32
    x = x ^ (x >> np.uint64(16))
    return x


def stream_key(seed: int, iteration: int, tensor: int) -> int:
    """Fold (seed, iteration, tensor index) into one 32-bit word."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    it = int(iteration) & 0xFFFFFFFFFFFFFFFF
    h = int(mix32((seed & _M32) ^ 0x9E3779B9))
    h = int(mix32(h ^ (seed >> 32)))
    h = int(mix32(h ^ (it & _M32)))
    h = int(mix32(h ^ (it >> 32)))
    h = int(mix32(h ^ (int(tensor) & _M32)))
    return h


def sample_positions(seed: int, iteration: int, tensor: int, plan: SamplePlan,
                     block: int) -> np.ndarray:
    """Element positions (relative to the tensor's start) of the sample.

    Draw q picks aligned block floor(r_q * nblocks / 2**32) with
    r_q = mix32(key ^ (q * 0x9E3779B1 mod 2**32)); the sample is every element
    of every drawn block, draws with replacement.
    """
    if plan.exact:
        return np.arange(plan.count, dtype=np.int64)
    key = stream_key(seed, iteration, tensor)
    q = np.arange(plan.blocks, dtype=np.uint64)
    r = mix32(np.uint64(key) ^ ((q * np.uint64(0x9E3779B1)) & _M32))
    blk = (r * np.uint64(plan.nblocks)) >> np.uint64(32)
    pos = blk[:, None] * np.uint64(block) + np.arange(block, dtype=np.uint64)[None, :]
    return pos.reshape(-1).astype(np.int64)


# --------------------------------------------------------------------------
# Threshold selection (Algorithm 3 "thr <- s% of |V[j]|"; Section 5)
# --------------------------------------------------------------------------
def select_threshold(magnitudes: np.ndarray, rank: int) -> np.float32:
    """Magnitude of 0-based descending rank `rank`; -1 if the set is too small."""
    if rank >= magnitudes.size:
        return np.float32(-1.0)
    ordered = np.sort(magnitudes.astype(np.float32))[::-1]
    return np.float32(ordered[rank])


# --------------------------------------------------------------------------
# One compression step of one worker (Algorithm 3 / 4, everything but the
# forward/backward pass and the exchange)
# --------------------------------------------------------------------------
@dataclass
class CompressResult:
    indices: List[np.ndarray]        # per tensor, ascending global flat indices (int32)
    values: List[np.ndarray]         # per tensor, the sent V values (float32)
    thresholds: np.ndarray           # per tensor (float32)
    counts: np.ndarray               # per tensor: how many passed the mask (int64)
    norm: float
    scale: np.float32
    overflow: bool = False
    refined: List[bool] = field(default_factory=list)


def compress(g: np.ndarray, u: np.ndarray, v: np.ndarray, offsets: Sequence[int],
             cfg: OracleConfig, iteration: int,
             capacities: Optional[Sequence[int]] = None) -> CompressResult:
    """Run one iteration on flat g, u, v (u and v are updated in place).

    `offsets` has one entry per tensor plus the total; tensor j is
    [offsets[j], offsets[j+1]).  `capacities[j]` bounds the pairs tensor j may
    emit: the lowest indices are kept, the rest is neither sent nor masked.
    """
    n = int(offsets[-1])
    assert g.shape == (n,) and u.shape == (n,) and v.shape == (n,)
    # -- clipping -----------------------------------------------------------
    norm = float("nan")
    scale = np.float32(1.0)
    if cfg.clip_threshold > 0.0:
        norm, scale = clip_scale(g, cfg.clip_threshold, cfg.num_workers)
    if cfg.scale_override is not None:
        scale = np.float32(cfg.scale_override)
    # -- momentum correction --------------------------------------------------
    u1, v1 = momentum_correction(g, u, v, cfg.momentum, scale, cfg.nesterov)
    # -- per-tensor threshold, mask, extract, clear ------------------------------
    T = len(offsets) - 1
    res = CompressResult([], [], np.zeros(T, np.float32), np.zeros(T, np.int64),
                         norm, scale)
    for j in range(T):
        lo, hi = int(offsets[j]), int(offsets[j + 1])
        nj = hi - lo
        vj = v1[lo:hi]
        mag = np.abs(vj)
        plan = sample_plan(nj, cfg)
        pos = sample_positions(cfg.seed, iteration, j, plan, cfg.sample_block)
        thr = select_threshold(mag[pos], plan.rank)
        keep = mag > thr
        refined = False
        if cfg.refine_alpha is not None and int(keep.sum()) > cfg.refine_alpha * plan.k:
            thr = select_threshold(mag[keep], plan.k)
            keep = mag > thr
            refined = True
        res.counts[j] = int(keep.sum())
        sel = np.flatnonzero(keep)
        if capacities is not None and sel.size > int(capacities[j]):
            sel = sel[: int(capacities[j])]
            res.overflow = True
        res.thresholds[j] = thr
        res.refined.append(refined)
        res.indices.append((sel + lo).astype(np.int32))
        res.values.append(vj[sel].copy())
        vj[sel] = np.float32(0.0)
        if cfg.factor_masking:
            u1[lo:hi][sel] = np.float32(0.0)
    u[:] = u1
    v[:] = v1
    return res


def flatten_payload(res: CompressResult) -> Tuple[np.ndarray, np.ndarray]:
    """All tensors' pairs as one ascending (index, value) list."""
    if not res.indices:
        return np.zeros(0, np.int32), np.zeros(0, np.float32)
    return np.concatenate(res.indices), np.concatenate(res.values)


# --------------------------------------------------------------------------
# Receive side (the sum in Algorithm 3's all-reduce line)
# --------------------------------------------------------------------------
def decompress_accumulate(dense: np.ndarray,
                          payloads: Sequence[Tuple[np.ndarray, np.ndarray]]) -> None:
    """dense[idx] += val for every pair, workers in the order given, binary32."""
    assert dense.dtype == np.float32
    for idx, val in payloads:
        np.add.at(dense, np.asarray(idx, dtype=np.int64), np.asarray(val, dtype=np.float32))


def sparse_sgd_apply(theta: np.ndarray, payloads: Sequence[Tuple[np.ndarray, np.ndarray]],
                     learning_rate: float) -> None:
    """Last line of Algorithm 3 with plain SGD, applied pair by pair:
    theta[idx] <- theta[idx] - lr * val, workers in the order given, binary32, the
    product rounded before the subtraction.  Equal to theta - lr * G_t (G_t the sum
    of the sparse gradients) up to rounding, and exactly where an index occurs once."""
    assert theta.dtype == np.float32
    lr = np.float32(learning_rate)
    for idx, val in payloads:
        step = lr * np.asarray(val, dtype=np.float32)
        np.subtract.at(theta, np.asarray(idx, dtype=np.int64), step)


# --------------------------------------------------------------------------
# Wire format (Section 3.1: "encode() packs the 32-bit nonzero gradient values
# and 16-bit run lengths of zeros"; Table 3 footnote)
# --------------------------------------------------------------------------
RUN_MAX = 65535
"""Largest zero-run a 16-bit field holds."""


def encode(indices: np.ndarray, values: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Entries (run, value) of the flattened sparse gradient, in index order.

    `run` zeros precede `value`.  The paper does not say what happens when more
    than 65535 zeros separate two values; the reading used here: an entry
    (65535, 0.0) stands for 65535 zeros followed by one explicit zero element,
    i.e. it advances 65536 positions, and as many of them as needed precede the
    real entry.  Trailing zeros are not encoded (the length is known)."""
    order = np.argsort(indices, kind="stable")
    idx = np.asarray(indices, dtype=np.int64)[order]
    val = np.asarray(values, dtype=np.float32)[order]
    runs: List[int] = []
    vals: List[np.float32] = []
    pos = 0                                  # next position not yet described
    for i, x in zip(idx.tolist(), val.tolist()):
        gap = i - pos
        assert gap >= 0, "indices must be distinct"
        while gap > RUN_MAX:
            runs.append(RUN_MAX)
            vals.append(np.float32(0.0))
            gap -= RUN_MAX + 1
        runs.append(gap)
        vals.append(np.float32(x))
        pos = i + 1
    return np.asarray(runs, dtype=np.uint16), np.asarray(vals, dtype=np.float32)


def decode_accumulate(dense: np.ndarray, runs: np.ndarray, vals: np.ndarray) -> None:
    """dense[position] += value for every entry, binary32, entries in order."""
    assert dense.dtype == np.float32
    pos = 0
    for r, x in zip(runs.tolist(), vals.tolist()):
        pos += r
        dense[pos] = dense[pos] + np.float32(x)
        pos += 1


def encoded_bytes(entries: int) -> int:
    """Six bytes per entry: a 32-bit value and a 16-bit run length."""
    return 6 * int(entries)


def compression_ratio(n: int, pairs: int, bytes_per_pair: int) -> float:
    """Dense bytes over payload bytes (the tables print this reciprocal of the
    formula of Section 4.1, e.g. 277x)."""
    return (4.0 * n) / (bytes_per_pair * pairs) if pairs else float("inf")
