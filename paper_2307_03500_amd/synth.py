"""Seeded synthetic gradient sets shaped like the models the paper trains.

This module only makes inputs: tensor-size lists and flat fp32 vectors.  It holds none of
the method's arithmetic (no partitioning, norms, budgets, packing or selection), so both the
CPU oracle's tests and the GPU path's tests/bench may draw their inputs from it.

The paper measures on gradients of ResNet-18 / CIFAR-10, an LSTM language model /
WikiText-2 and NCF / MovieLens-20M (Table 2).  Neither those datasets nor trained gradients
are used here: each config below takes the tensor shapes of an architecture (hyper-parameters
only) and fills them with a seeded per-tensor distribution.

Reproducibility: every block of at most ``_BLOCK`` elements of every tensor is drawn from its
own Philox stream keyed by (seed, tensor index, block index), so the result does not depend
on the number of threads used to fill the vector.
"""
from __future__ import annotations

import concurrent.futures as _cf
import os as _os
from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence

import numpy as np

_BLOCK = 1 << 22  # elements per independently-seeded block


# --------------------------------------------------------------------------------------
# tensor-size lists (model order)
# --------------------------------------------------------------------------------------
def toy_mlp_sizes() -> List[int]:
    """784-256-256-128-10 MLP: weight, bias per layer."""
    return [784 * 256, 256, 256 * 256, 256, 256 * 128, 128, 128 * 10, 10]


def resnet18_sizes() -> List[int]:
    """ImageNet-style ResNet-18: 62 tensors, 11 689 512 parameters."""
    s: List[int] = [64 * 3 * 7 * 7, 64, 64]
    cin = 64
    for c in (64, 128, 256, 512):
        for block in range(2):
            first = block == 0 and c != 64
            s += [c * (cin if block == 0 else c) * 9, c, c, c * c * 9, c, c]
            if first:
                s += [c * cin, c, c]  # 1x1 downsample conv + its BN pair
        cin = c
    s += [1000 * 512, 1000]
    return s


def lstm_lm_sizes() -> List[int]:
    """2-layer LSTM LM: vocab 10000, hidden 650, untied decoder."""
    v, h = 10000, 650
    s = [v * h]
    for _ in range(2):
        s += [4 * h * h, 4 * h * h, 4 * h, 4 * h]
    s += [v * h, v]
    return s


def bert_base_sizes() -> List[int]:
    """BERT-base: 199 tensors, 109 482 240 parameters."""
    h, ff, v = 768, 3072, 30522
    s = [v * h, 512 * h, 2 * h, h, h]
    for _ in range(12):
        s += [h * h, h] * 4  # Q, K, V, O
        s += [h, h]  # attention LayerNorm
        s += [ff * h, ff, h * ff, h]
        s += [h, h]  # output LayerNorm
    s += [h * h, h]  # pooler
    return s


def gpt2_medium_sizes() -> List[int]:
    """GPT-2 medium: 292 tensors, 354 823 168 parameters."""
    h, ff, v, ctx = 1024, 4096, 50257, 1024
    s = [v * h, ctx * h]
    for _ in range(24):
        s += [h, h, h * 3 * h, 3 * h, h * h, h, h, h, h * ff, ff, ff * h, h]
    s += [h, h]
    return s


def ncf_sizes() -> List[int]:
    """Neural collaborative filtering sized like MovieLens-20M (138 493 users, 26 744 items):
    GMF embeddings of width 64, MLP embeddings of width 128, MLP 256-256-128-64, output 128-1.
    The paper gives no NCF shapes (Table 2 names only the model); these are this build's."""
    users, items = 138493, 26744
    s = [users * 64, items * 64, users * 128, items * 128]
    for a, b in ((256, 256), (256, 128), (128, 64)):
        s += [a * b, b]
    s += [128, 1]
    return s


# --------------------------------------------------------------------------------------
# value fills
# --------------------------------------------------------------------------------------
def _rng(seed: int, tensor: int, block: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), (tensor << 24) | block]))


def _fill_normal(rng, out, scale):
    out[:] = rng.standard_normal(out.shape[0], dtype=np.float32) * np.float32(scale)


def _fill_laplace(rng, out, scale):
    out[:] = rng.laplace(0.0, scale, out.shape[0]).astype(np.float32)


def _fill_student3(rng, out, scale):
    out[:] = (rng.standard_t(3.0, out.shape[0]) * scale).astype(np.float32)


def _round_through_bf16(x: np.ndarray) -> None:
    """fp32 -> bf16 (round to nearest, ties to even) -> fp32, in place."""
    u = x.view(np.uint32)
    u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    u &= np.uint32(0xFFFF0000)


@dataclass
class GradientSet:
    name: str
    tensor_sizes: List[int]
    g: np.ndarray  # flat fp32, len = sum(tensor_sizes)
    d: float
    n_workers: int
    seed: int

    @property
    def N(self) -> int:
        return int(self.g.shape[0])


@dataclass
class _Recipe:
    sizes: Callable[[], List[int]]
    fill: Callable
    log10_scale: Sequence[float]
    d: float
    n_workers: int
    bf16: bool = False
    zero_rows: Optional[tuple] = None  # (tensor index, rows, cols, rows kept non-zero)


CONFIGS = {
    "toy_mlp": _Recipe(toy_mlp_sizes, _fill_normal, (-4.0, -1.0), 0.01, 4),
    "resnet18": _Recipe(resnet18_sizes, _fill_normal, (-5.0, -1.0), 0.01, 16),
    "lstm_lm": _Recipe(lstm_lm_sizes, _fill_laplace, (-4.0, -1.0), 0.001, 8,
                       zero_rows=(0, 10000, 650, 1000)),
    "bert_base": _Recipe(bert_base_sizes, _fill_student3, (-5.0, -1.0), 0.01, 16),
    "gpt2_medium": _Recipe(gpt2_medium_sizes, _fill_student3, (-5.0, -1.0), 0.001, 32, bf16=True),
    # dense selection (d = 0.1, the density the paper uses for NCF in Sec. 5.2); embedding rows
    # of inactive users/items carry no gradient: 70 % of the rows of each table are exactly 0
    "ncf": _Recipe(ncf_sizes, _fill_laplace, (-4.0, -1.0), 0.1, 16,
                   zero_rows=((0, 138493, 64, 41548), (1, 26744, 64, 8023),
                              (2, 138493, 128, 41548), (3, 26744, 128, 8023))),
}


def tensor_sizes(name: str) -> List[int]:
    return CONFIGS[name].sizes()


def make(name: str, seed: int = 0, threads: Optional[int] = None) -> GradientSet:
    """Build the named gradient set.  Deterministic in (name, seed)."""
    r = CONFIGS[name]
    sizes = r.sizes()
    N = int(sum(sizes))
    g = np.empty(N, dtype=np.float32)
    lo, hi = r.log10_scale
    scales = 10.0 ** _rng(seed, (1 << 30), 0).uniform(lo, hi, len(sizes))

    jobs = []
    pos = 0
    for t, s in enumerate(sizes):
        for b, st in enumerate(range(0, s, _BLOCK)):
            jobs.append((t, b, pos + st, min(_BLOCK, s - st)))
        pos += s

    def run(job):
        t, b, st, ln = job
        view = g[st:st + ln]
        r.fill(_rng(seed, t, b), view, float(scales[t]))
        if r.bf16:
            _round_through_bf16(view)

    if threads is None:
        threads = min(16, len(_os.sched_getaffinity(0)))
    if threads > 1 and len(jobs) > 1:
        with _cf.ThreadPoolExecutor(threads) as ex:
            list(ex.map(run, jobs))
    else:
        for j in jobs:
            run(j)

    if r.zero_rows is not None:
        specs = r.zero_rows if isinstance(r.zero_rows[0], tuple) else (r.zero_rows,)
        for i, (t, rows, cols, keep) in enumerate(specs):
            st = int(sum(sizes[:t]))
            perm = _rng(seed, (1 << 30) + 1 + i, 0).permutation(rows)
            zero = np.sort(perm[keep:])
            g[st:st + rows * cols].reshape(rows, cols)[zero, :] = 0.0
    return GradientSet(name, sizes, g, r.d, r.n_workers, seed)


def random_layers(seed: int, n_layers: int, max_size: int, kind: str = "normal",
                  tie_levels: int = 0):
    """Small ragged test inputs: (sizes, g).  ``tie_levels`` > 0 quantises |g| to that many
    distinct magnitudes so that equal-|g| ties are everywhere."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xABCD]))
    sizes = [int(x) for x in rng.integers(1, max_size + 1, n_layers)]
    N = sum(sizes)
    if kind == "normal":
        g = rng.standard_normal(N).astype(np.float32)
    elif kind == "student":
        g = rng.standard_t(3.0, N).astype(np.float32)
    else:
        raise ValueError(kind)
    pos = 0
    for s in sizes:
        g[pos:pos + s] *= np.float32(10.0 ** rng.uniform(-4, 0))
        pos += s
    if tie_levels > 0:
        sign = np.where(rng.integers(0, 2, N) == 0, -1.0, 1.0).astype(np.float32)
        g = (rng.integers(0, tie_levels, N).astype(np.float32) * np.float32(0.125)) * sign
    return sizes, g
