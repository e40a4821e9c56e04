"""Seeded synthetic gradient sets shaped like the paper's models.

This module only lists tensor shapes and draws random numbers.  It holds none
of the method's arithmetic, so both the HIP path's callers and the CPU oracle's
callers may feed from it.  The gradients stand in for those of the paper's
ImageNet, Penn Treebank and LibriSpeech runs (Tables 3 and 4), whose data and
trained weights are not available: shapes and sizes follow the models named
there, values are heavy-tailed noise (Student-t, 3 degrees of freedom) with a
per-tensor scale drawn log-uniformly in [1e-5, 1e-2].
"""

from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]

    @property
    def numel(self) -> int:
        return int(math.prod(self.shape))


@dataclass(frozen=True)
class GradientSet:
    name: str
    tensors: Tuple[TensorSpec, ...]

    @property
    def sizes(self) -> List[int]:
        return [t.numel for t in self.tensors]

    @property
    def offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.sizes)]).astype(np.int64)

    @property
    def numel(self) -> int:
        return int(sum(self.sizes))


# ---------------------------------------------------------------------------
# Manifests
# ---------------------------------------------------------------------------
def toy_set(n: int = 1 << 20) -> GradientSet:
    return GradientSet("toy", (TensorSpec("w", (n,)),))


def resnet50_set() -> GradientSet:
    """161 tensors, 25,557,032 parameters = 97.49 MiB (Table 3's baseline size)."""
    ts: List[TensorSpec] = []

    def bn(prefix: str, c: int) -> None:
        ts.append(TensorSpec(prefix + ".weight", (c,)))
        ts.append(TensorSpec(prefix + ".bias", (c,)))

    ts.append(TensorSpec("conv1.weight", (64, 3, 7, 7)))
    bn("bn1", 64)
    inplanes = 64
    for stage, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3)), 1):
        for b in range(blocks):
            p = f"layer{stage}.{b}"
            ts.append(TensorSpec(p + ".conv1.weight", (planes, inplanes, 1, 1)))
            bn(p + ".bn1", planes)
            ts.append(TensorSpec(p + ".conv2.weight", (planes, planes, 3, 3)))
            bn(p + ".bn2", planes)
            ts.append(TensorSpec(p + ".conv3.weight", (planes * 4, planes, 1, 1)))
            bn(p + ".bn3", planes * 4)
            if b == 0:
                ts.append(TensorSpec(p + ".downsample.0.weight", (planes * 4, inplanes, 1, 1)))
                bn(p + ".downsample.1", planes * 4)
            inplanes = planes * 4
    ts.append(TensorSpec("fc.weight", (1000, 2048)))
    ts.append(TensorSpec("fc.bias", (1000,)))
    return GradientSet("resnet50", tuple(ts))


LSTM_EMBED_ROWS = 10000
LSTM_EMBED_DIM = 1500
LSTM_ACTIVE_ROWS = 700


def lstm_lm_set() -> GradientSet:
    """Untied 2-layer LSTM-1500 language model, 66,034,000 parameters."""
    ts = [TensorSpec("encoder.weight", (LSTM_EMBED_ROWS, LSTM_EMBED_DIM))]
    for l in range(2):
        ts.append(TensorSpec(f"rnn.weight_ih_l{l}", (6000, 1500)))
        ts.append(TensorSpec(f"rnn.weight_hh_l{l}", (6000, 1500)))
        ts.append(TensorSpec(f"rnn.bias_ih_l{l}", (6000,)))
        ts.append(TensorSpec(f"rnn.bias_hh_l{l}", (6000,)))
    ts.append(TensorSpec("decoder.weight", (10000, 1500)))
    ts.append(TensorSpec("decoder.bias", (10000,)))
    return GradientSet("lstm_lm", tuple(ts))


def speech_set() -> GradientSet:
    """Two convolutions, seven bidirectional GRU layers of 1200 units
    (Section 4.1's speech model), one output layer: 122,153,069 parameters."""
    ts = [TensorSpec("conv.0.weight", (32, 1, 41, 11)), TensorSpec("conv.0.bias", (32,)),
          TensorSpec("conv.1.weight", (32, 32, 21, 11)), TensorSpec("conv.1.bias", (32,))]
    hidden = 1200
    for l in range(7):
        inp = 1312 if l == 0 else hidden
        for d in ("", "_reverse"):
            ts.append(TensorSpec(f"gru.{l}.weight_ih{d}", (3 * hidden, inp)))
            ts.append(TensorSpec(f"gru.{l}.weight_hh{d}", (3 * hidden, hidden)))
            ts.append(TensorSpec(f"gru.{l}.bias_ih{d}", (3 * hidden,)))
            ts.append(TensorSpec(f"gru.{l}.bias_hh{d}", (3 * hidden,)))
    ts.append(TensorSpec("fc.weight", (29, hidden)))
    ts.append(TensorSpec("fc.bias", (29,)))
    return GradientSet("speech", tuple(ts))


def speech_literal_set() -> GradientSet:
    """The speech set read literally from the shapes of the benchmark description: two
    convolutions, five bidirectional GRU layers of 1024 units (directions concatenated, 1312
    input features), an output layer of 1024 x 29: 90,192,061 parameters, which is short of
    the 488 MB the paper prints for its model (Table 4); `speech_set` is the one that meets it."""
    ts = [TensorSpec("conv.0.weight", (32, 1, 41, 11)), TensorSpec("conv.0.bias", (32,)),
          TensorSpec("conv.1.weight", (32, 32, 21, 11)), TensorSpec("conv.1.bias", (32,))]
    hidden = 1024
    for l in range(5):
        inp = 1312 if l == 0 else 2 * hidden
        for d in ("", "_reverse"):
            ts.append(TensorSpec(f"gru.{l}.weight_ih{d}", (3 * hidden, inp)))
            ts.append(TensorSpec(f"gru.{l}.weight_hh{d}", (3 * hidden, hidden)))
            ts.append(TensorSpec(f"gru.{l}.bias_ih{d}", (3 * hidden,)))
            ts.append(TensorSpec(f"gru.{l}.bias_hh{d}", (3 * hidden,)))
    ts.append(TensorSpec("fc.weight", (29, hidden)))
    ts.append(TensorSpec("fc.bias", (29,)))
    return GradientSet("speech_literal", tuple(ts))


def ragged_set(seed: int = 0, tensors: int = 23, max_numel: int = 70000) -> GradientSet:
    """Small set with odd sizes (tiny, unaligned and multi-tile tensors)."""
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed), 77])))
    sizes = [1, 3, 29, 64, 4097, 5000, 16384, 33333]
    while len(sizes) < tensors:
        sizes.append(int(math.exp(rng.uniform(0.0, math.log(max_numel)))))
    order = rng.permutation(len(sizes))
    return GradientSet("ragged", tuple(TensorSpec(f"t{i}", (int(sizes[i]),)) for i in order))


# ---------------------------------------------------------------------------
# Values
# ---------------------------------------------------------------------------
_CHUNK = 1 << 20


def _chunk_rng(base_seed: int, worker: int, iteration: int, salt: int, chunk: int) -> np.random.Generator:
    ss = np.random.SeedSequence([int(base_seed) & 0xFFFFFFFF, int(worker) & 0xFFFFFFFF,
                                 int(iteration) & 0xFFFFFFFF, int(salt), int(chunk)])
    return np.random.Generator(np.random.SFC64(ss))


def _fill_chunk(out: np.ndarray, base_seed: int, worker: int, iteration: int, salt: int, chunk: int) -> None:
    lo = chunk * _CHUNK
    hi = min(out.size, lo + _CHUNK)
    rng = _chunk_rng(base_seed, worker, iteration, salt, chunk)
    z = rng.standard_normal(hi - lo, dtype=np.float32)
    c = rng.standard_gamma(1.5, size=hi - lo, dtype=np.float32)
    # Student-t with 3 degrees of freedom: normal / sqrt(chi-square_3 / 3), chi-square_3 = 2 Gamma(3/2)
    np.maximum(c, np.float32(1e-20), out=c)      # keeps every draw finite
    np.multiply(c, np.float32(2.0 / 3.0), out=c)
    np.sqrt(c, out=c)
    np.divide(z, c, out=out[lo:hi])


def student_t3(n: int, base_seed: int, worker: int, iteration: int, salt: int = 0,
               out: Optional[np.ndarray] = None) -> np.ndarray:
    """n seeded fp32 draws of Student-t(3).  The stream is cut into fixed chunks with
    one generator each, so the values do not depend on how many threads fill them."""
    if out is None:
        out = np.empty(n, dtype=np.float32)
    chunks = (n + _CHUNK - 1) // _CHUNK
    workers = max(1, min(16, os.cpu_count() or 1, chunks))
    if workers == 1:
        for c in range(chunks):
            _fill_chunk(out, base_seed, worker, iteration, salt, c)
    else:
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda c: _fill_chunk(out, base_seed, worker, iteration, salt, c), range(chunks)))
    return out


def tensor_scales(gs: GradientSet, base_seed: int, fixed: Optional[float] = None) -> np.ndarray:
    """Per-tensor standard deviation, log-uniform in [1e-5, 1e-2], drawn once per set."""
    if fixed is not None:
        return np.full(len(gs.tensors), fixed, dtype=np.float64)
    rng = _chunk_rng(base_seed, 0xFFFF, 0xFFFF, 1, 0)
    return np.exp(rng.uniform(math.log(1e-5), math.log(1e-2), size=len(gs.tensors)))


def gradient(gs: GradientSet, base_seed: int, worker: int, iteration: int,
             scales: Optional[np.ndarray] = None, out: Optional[np.ndarray] = None) -> np.ndarray:
    """Flat fp32 gradient of worker `worker` at `iteration`: sigma_j * t(3) per tensor."""
    if scales is None:
        scales = tensor_scales(gs, base_seed)
    out = student_t3(gs.numel, base_seed, worker, iteration, 0, out)
    offs = gs.offsets
    for j in range(len(gs.tensors)):
        out[offs[j]:offs[j + 1]] *= np.float32(scales[j])
    return out


def toy_gradient(n: int, base_seed: int, worker: int, iteration: int) -> np.ndarray:
    """Toy configuration: 1e-3 * t(3)."""
    out = student_t3(n, base_seed, worker, iteration)
    out *= np.float32(1e-3)
    return out


def embedding_active_rows(base_seed: int, worker: int, iteration: int) -> np.ndarray:
    """Boolean mask over the 10000 embedding rows: the 700 seeded rows a step touches."""
    rng = _chunk_rng(base_seed, worker, iteration, 2, 0)
    rows = rng.choice(LSTM_EMBED_ROWS, size=LSTM_ACTIVE_ROWS, replace=False)
    keep = np.zeros(LSTM_EMBED_ROWS, dtype=bool)
    keep[rows] = True
    return keep


def zero_inactive_embedding_rows(g: np.ndarray, base_seed: int, worker: int, iteration: int) -> np.ndarray:
    """In place: the embedding gradient (first tensor of the LSTM set) is zero outside the active rows."""
    keep = embedding_active_rows(base_seed, worker, iteration)
    emb = g[: LSTM_EMBED_ROWS * LSTM_EMBED_DIM].reshape(LSTM_EMBED_ROWS, LSTM_EMBED_DIM)
    emb[~keep] = 0.0
    return g


def lstm_gradient(gs: GradientSet, base_seed: int, worker: int, iteration: int,
                  scales: Optional[np.ndarray] = None) -> np.ndarray:
    """As `gradient`, but the embedding gradient is zero outside 700 seeded rows."""
    g = gradient(gs, base_seed, worker, iteration, scales)
    return zero_inactive_embedding_rows(g, base_seed, worker, iteration)


def correlated_gradient(gs: GradientSet, base_seed: int, worker: int, iteration: int,
                        shared: np.ndarray, mix: float = 0.45,
                        scales: Optional[np.ndarray] = None) -> np.ndarray:
    """Worker gradient = mix * shared + (1 - mix) * private, both heavy-tailed, so
    that different workers' largest elements partly coincide."""
    private = gradient(gs, base_seed, worker + 1000, iteration, scales)
    private *= np.float32(1.0 - mix)
    private += np.float32(mix) * shared
    return private


def topk_overlap(idx_a: np.ndarray, idx_b: np.ndarray) -> float:
    """Fraction of a's indices also present in b."""
    if idx_a.size == 0:
        return 0.0
    return float(np.intersect1d(idx_a, idx_b).size) / float(idx_a.size)
