"""CPU oracle for DEFT's gradient-selection path (Yoon & Oh, ICPP 2023).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct statement of what
the GPU library must compute.  Only tests/, the smoke check and the bench's cpu_baseline leg
may import it; the product package never does, and this file imports nothing from the
product.  It shares no code, tables or helpers with the HIP path.

Each function cites the passage of the paper it follows.  The planner steps (Alg. 2, 3, 4)
are heuristics with no independent "true answer", so they are written out step by step in
the paper's order and notation.  The selection steps (Alg. 5 and the conventional Top-k of
Sec. 1 / 3.1) have a plain definition -- sort by magnitude, keep the first k -- and the
oracle is that definition.

Readings taken where the paper is silent:
  * norm = L2 norm, plain (not squared)                               (Sec. 4.2; Sec. 2 uses L2)
  * k = n_g * d is rounded half-up to an integer:  K = floor(N*d + 0.5)      (Alg. 3, first step)
  * priority = norm descending, ties by layer position ascending             (Sec. 4.2)
  * norm_remain at each step is the sum of the norms of the layers not yet served,
    accumulated from the last-priority layer backwards (same quantity as the running
    subtraction of Alg. 3, without its floating-point drift)
  * k_temp is truncated (floor) to an integer
  * log is the natural logarithm                                              (Eq. 3)
  * argmax / argmin ties: first occurrence in positional layer order / lowest bin id (Alg. 4)
  * equal |g|: the lower index wins; a segment's picks are listed by ascending index
  * magnitudes are compared through the integer key  bits(g) & 0x7fffffff, which orders
    |g| exactly for every non-NaN float, makes -0 == +0 and ranks NaN above inf.

All floating-point steps are IEEE fp64 with no fused multiply-add.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

__all__ = [
    "partition", "layer_sumsq", "layer_norms", "total_k", "alloc_k", "layer_costs",
    "assign_layers", "magnitude_key", "topk_segment", "select", "topk_global", "cost_model",
    "accumulate", "gather_zero",
]


# --------------------------------------------------------------------------------------
# Alg. 2 -- two-stage gradient vector partitioning (Sec. 4.1)
# --------------------------------------------------------------------------------------
def partition(tensor_sizes: Sequence[int], n_workers: int) -> Tuple[List[int], List[int]]:
    """Return (offsets, layer_tensor).  offsets has L+1 entries; layer l is
    [offsets[l], offsets[l+1]).  layer_tensor[l] is the index of the tensor it came from.

    A tensor larger than n_g / n_workers is cut into n_workers contiguous fractions whose
    sizes differ by at most one, the larger ones first (Alg. 2, second stage).  Empty
    tensors and empty fractions produce no layer.
    """
    if n_workers < 1:
        raise ValueError("n_workers must be >= 1")
    sizes = [int(s) for s in tensor_sizes]
    if any(s < 0 for s in sizes):
        raise ValueError("negative tensor size")
    n_g = sum(sizes)
    # the pieces every tensor contributes, in model order
    pieces: List[Tuple[int, int]] = []  # (tensor index, piece size)
    for t, size in enumerate(sizes):
        # "larger than n_g / n_workers", decided exactly in integers
        if size * n_workers > n_g:
            small, extra = divmod(size, n_workers)
            # `extra` pieces of small + 1 elements come first, then pieces of `small`
            cut = [small + 1] * extra + [small] * (n_workers - extra)
        else:
            cut = [size]
        pieces.extend((t, c) for c in cut if c > 0)
    offsets = [0]
    for _, c in pieces:
        offsets.append(offsets[-1] + c)
    return offsets, [t for t, _ in pieces]


# --------------------------------------------------------------------------------------
# Sec. 4.2 -- gradient norm of each layer
# --------------------------------------------------------------------------------------
_NORM_BLOCK = 1 << 16


def layer_sumsq(g: np.ndarray, offsets: Sequence[int]) -> np.ndarray:
    """Sum of squares of each layer in fp64.  Each fp32 value is widened to fp64 (its square
    is then exact), block sums use numpy's pairwise fp64 summation and the block sums are
    combined with math.fsum (correctly rounded), so the result is within a few ulp of the
    exact value."""
    L = len(offsets) - 1
    out = np.zeros(L, dtype=np.float64)
    for l in range(L):
        s, e = int(offsets[l]), int(offsets[l + 1])
        parts = []
        for b in range(s, e, _NORM_BLOCK):
            x = g[b:min(e, b + _NORM_BLOCK)].astype(np.float64)
            parts.append(float(np.sum(x * x)))
        out[l] = math.fsum(parts)
    return out


def layer_norms(g: np.ndarray, offsets: Sequence[int]) -> np.ndarray:
    """L2 norm of each layer (Sec. 4.2: the gradient norm of each layer sets its priority)."""
    return np.sqrt(layer_sumsq(g, offsets))


# --------------------------------------------------------------------------------------
# Alg. 3 -- gradient-norm-based local k assignment (Sec. 4.2)
# --------------------------------------------------------------------------------------
def total_k(n_g: int, d: float) -> int:
    """k = n_g * d (footnote on density in Sec. 1; first step of Alg. 3), rounded half-up."""
    return int(math.floor(float(n_g) * float(d) + 0.5))


def alloc_k(norms: Sequence[float], sizes: Sequence[int], n_g: int, d: float) -> List[int]:
    """Local k of every layer, indexed by layer position.

    Layers are served in priority order (largest norm first).  Each takes the share
    k_remain * norm / norm_remain of what is left, capped by its size and never below 1;
    k_remain is then reduced by what it took (Alg. 3)."""
    L = len(sizes)
    if len(norms) != L:
        raise ValueError("norms and sizes differ in length")
    norm = [float(x) for x in norms]
    order = sorted(range(L), key=lambda l: (-norm[l], l))
    # norm_remain[j] = sum of norms of order[j:], accumulated from the back
    norm_remain = [0.0] * L
    acc = 0.0
    for j in range(L - 1, -1, -1):
        acc = norm[order[j]] + acc
        norm_remain[j] = acc
    k_remain = total_k(n_g, d)
    k = [0] * L
    for j, l in enumerate(order):
        if norm_remain[j] > 0.0:
            k_temp = float(k_remain) * (norm[l] / norm_remain[j])
        else:
            k_temp = 0.0
        size = int(sizes[l])
        if size < k_temp:
            k_l = size
        else:
            k_l = max(1, int(math.floor(k_temp)))
        k[l] = k_l
        k_remain -= k_l
    return k


# --------------------------------------------------------------------------------------
# Alg. 4 -- bin-packing-based layer allocation (Sec. 4.3, Eq. 3)
# --------------------------------------------------------------------------------------
def layer_costs(sizes: Sequence[int], k: Sequence[int]) -> List[float]:
    """c_x = n_{g,x} * log k_x  (Eq. 3)."""
    return [float(int(s)) * math.log(float(int(kk))) for s, kk in zip(sizes, k)]


def assign_layers(sizes: Sequence[int], k: Sequence[int], n_workers: int, iteration: int,
                  rank: int) -> Tuple[List[int], List[int], List[List[int]]]:
    """Return (owner_bin, alloc_part, alloc_bin).

    Repeatedly take the most expensive unplaced layer and put it into the currently lightest
    bin (Sec. 4.3).  The worker's bin is (iteration % n + rank) % n.  Every caller plays the
    delegate: the broadcast of Alg. 4 is not part of a one-GPU run."""
    if n_workers < 1 or not (0 <= rank < n_workers) or iteration < 0:
        raise ValueError("bad n_workers / rank / iteration")
    L = len(sizes)
    cost = layer_costs(sizes, k)
    load = [0.0] * n_workers                      # summed cost of each bin so far
    alloc_bin: List[List[int]] = [[] for _ in range(n_workers)]
    unplaced = list(range(L))
    while unplaced:
        # most expensive layer still unplaced; among equals the one that comes first
        layer = max(unplaced, key=lambda l: (cost[l], -l))
        # lightest bin; among equals the lowest id
        target = min(range(n_workers), key=lambda b: (load[b], b))
        alloc_bin[target].append(layer)
        load[target] = load[target] + cost[layer]
        unplaced.remove(layer)
    owner_bin = [0] * L
    for b, members in enumerate(alloc_bin):
        for l in members:
            owner_bin[l] = b
    mine = (iteration % n_workers + rank) % n_workers
    return owner_bin, list(alloc_bin[mine]), alloc_bin


# --------------------------------------------------------------------------------------
# Alg. 5 -- layer-wise gradient selection (Sec. 4.4), and the conventional Top-k (Sec. 1)
# --------------------------------------------------------------------------------------
def magnitude_key(x: np.ndarray) -> np.ndarray:
    """Integer that orders |x|: the fp32 bit pattern with the sign bit cleared."""
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def topk_segment(x: np.ndarray, k: int) -> np.ndarray:
    """Local indices (ascending) of the k entries of x with the largest magnitude; among
    equal magnitudes the lower index is preferred.  Definition by full sort."""
    n = int(x.shape[0])
    if not (0 <= k <= n):
        raise ValueError("k out of range")
    key = magnitude_key(x).astype(np.int64)
    # stable ascending sort of -key == key descending, index ascending among equals
    order = np.argsort(-key, kind="stable")
    picks = order[:k]
    return np.sort(picks)


def select(g: np.ndarray, offsets: Sequence[int], k: Sequence[int],
           alloc_part: Sequence[int]) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Alg. 5: for each allocated layer, Top-k_l by magnitude, shifted by the layer's start.
    Returns (indices int64, values fp32, seg_off int64[len(alloc_part)+1])."""
    idx_parts, seg_off = [], [0]
    for part in alloc_part:
        s, e = int(offsets[part]), int(offsets[part + 1])
        part_idx = topk_segment(g[s:e], int(k[part])) + s
        idx_parts.append(part_idx)
        seg_off.append(seg_off[-1] + int(k[part]))
    idx = np.concatenate(idx_parts).astype(np.int64) if idx_parts else np.zeros(0, np.int64)
    return idx, g[idx], np.asarray(seg_off, dtype=np.int64)


def topk_global(g: np.ndarray, K: int) -> Tuple[np.ndarray, np.ndarray]:
    """Conventional Top-k sparsifier: the K largest-magnitude entries of the whole vector
    (Sec. 1; the n = 1 case of Sec. 5.4)."""
    idx = topk_segment(g, K).astype(np.int64)
    return idx, g[idx]


# --------------------------------------------------------------------------------------
# Eq. 4-9 -- selection cost model
# --------------------------------------------------------------------------------------
def cost_model(sizes: Sequence[int], k: Sequence[int], alloc_bin: Sequence[Sequence[int]],
               n_g: int, K: int) -> dict:
    """C_i (Eq. 4), C(n) (Eq. 5), f(n) (Eq. 6), C_trivial (Eq. 7), f_trivial (Eq. 8)."""
    n = len(alloc_bin)
    c = layer_costs(sizes, k)
    C_i = [math.fsum(c[l] for l in lst) for lst in alloc_bin]
    C_n = max(C_i)
    topk_cost = float(n_g) * math.log(float(K)) if K > 0 else 0.0
    C_triv = (float(n_g) / n) * math.log(float(K) / n) if K > n else 0.0
    return {
        "C_i": C_i,
        "C_n": C_n,
        "f_n": topk_cost / C_n if C_n > 0 else math.inf,
        "C_trivial": C_triv,
        "f_trivial": topk_cost / C_triv if C_triv > 0 else math.inf,
    }


# --------------------------------------------------------------------------------------
# Alg. 1 -- the steps around the sparsifier (error feedback)
# --------------------------------------------------------------------------------------
def accumulate(e: np.ndarray, grad: np.ndarray, eta: float) -> np.ndarray:
    """acc = e + eta * G  (Alg. 1, the step before Sparsify), in fp32 like the vectors
    themselves: the product is rounded to fp32, then the sum is rounded to fp32 (two separate
    operations, no fused multiply-add)."""
    e = np.ascontiguousarray(e, dtype=np.float32)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    prod = np.multiply(grad, np.float32(eta), dtype=np.float32)
    return np.add(e, prod, dtype=np.float32)


def gather_zero(acc: np.ndarray, idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """g_i = acc[idx]; acc[idx] = 0; e_next = acc  (Alg. 1, the steps after the index
    exchange).  idx holds distinct positions.  Returns (values, e_next); acc is not modified."""
    idx = np.asarray(idx, dtype=np.int64)
    vals = acc[idx].copy()
    e_next = acc.copy()
    e_next[idx] = np.float32(0.0)
    return vals, e_next
