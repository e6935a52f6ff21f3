"""One worker's DEFT sparsifier (Sec. 4 of the paper) as a sequence of C-ABI calls.

This class only owns buffers and orders the calls; it computes nothing itself:
  deft_partition (once) -> deft_layer_norms [device] -> stream sync ->
  deft_norms_from_sumsq -> deft_alloc_k -> deft_assign_layers [host] -> deft_select [device].
torch supplies device memory, pinned host memory and the stream.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np
import torch

from . import binding as B


@dataclass
class Selection:
    norms: np.ndarray       # L2 norm per layer (host)
    k: np.ndarray           # local k per layer (host)
    owner_bin: np.ndarray   # bin of each layer (host)
    my_layers: np.ndarray   # this worker's layers, in placement order (host)
    seg_off: np.ndarray     # output segment offsets (host)
    idx_dev: torch.Tensor   # int32 [k_r] global indices, device
    val_dev: torch.Tensor   # float32 [k_r] values, device
    times: dict = field(default_factory=dict)

    @property
    def idx(self) -> np.ndarray:
        return self.idx_dev.cpu().numpy()

    @property
    def val(self) -> np.ndarray:
        return self.val_dev.cpu().numpy()


class DeftSelector:
    def __init__(self, tensor_sizes: Sequence[int], n_workers: int, d: float, device,
                 out_cap: Optional[int] = None):
        self.device = torch.device(device)
        self.n = int(n_workers)
        self.d = float(d)
        self.offsets, self.layer_tensor = B.deft_partition(tensor_sizes, n_workers)
        self.L = len(self.offsets) - 1
        self.N = int(self.offsets[-1])
        self.sizes = np.diff(self.offsets).astype(np.int64)
        self.K = int(np.floor(self.N * self.d + 0.5))
        dev = self.device
        self.offsets_dev = torch.from_numpy(self.offsets).to(dev)
        self.sumsq_host = torch.zeros(self.L, dtype=torch.float64).pin_memory()
        nb = max(B.deft_workspace_bytes(B.OP_NORMS, self.N, self.L),
                 B.deft_workspace_bytes(B.OP_SELECT, self.N, self.L),
                 B.deft_workspace_bytes(B.OP_TOPK_GLOBAL, self.N, 1))
        self.ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        # sum of k_l can exceed K by the number of layers clamped up to 1 (Alg. 3)
        self.out_cap = int(out_cap) if out_cap is not None else self.K + self.L + 1
        self.idx_out = torch.empty(max(self.out_cap, self.K, 1), dtype=torch.int32, device=dev)
        self.val_out = torch.empty(max(self.out_cap, self.K, 1), dtype=torch.float32, device=dev)

    # -- steps ----------------------------------------------------------------------------
    def norms(self, g: torch.Tensor) -> np.ndarray:
        B.deft_layer_norms(g, self.offsets_dev, self.sumsq_host, self.ws)
        torch.cuda.current_stream().synchronize()
        return B.deft_norms_from_sumsq(self.sumsq_host.numpy())

    def plan(self, norms: np.ndarray, rank: int, iteration: int):
        k = B.deft_alloc_k(norms, self.sizes, self.N, self.d)
        owner, mine = B.deft_assign_layers(self.sizes, k, self.n, iteration, rank)
        return k, owner, mine

    def select(self, g: torch.Tensor, rank: int, iteration: int = 0, timed: bool = False) -> Selection:
        assert g.dtype == torch.float32 and g.numel() == self.N and g.device == self.device
        t0 = time.perf_counter()
        norms = self.norms(g)
        t1 = time.perf_counter()
        k, owner, mine = self.plan(norms, rank, iteration)
        t2 = time.perf_counter()
        seg = B.deft_select(g, self.offsets, k, mine, self.idx_out, self.val_out, self.ws)
        if timed:
            torch.cuda.current_stream().synchronize()
        t3 = time.perf_counter()
        kr = int(seg[-1])
        return Selection(norms, k, owner, mine, seg, self.idx_out[:kr], self.val_out[:kr],
                         {"norm_ms": (t1 - t0) * 1e3, "plan_ms": (t2 - t1) * 1e3,
                          "select_ms": (t3 - t2) * 1e3})

    def select_with_plan(self, g: torch.Tensor, k: np.ndarray, my_layers: np.ndarray):
        """Alg. 5 alone, for a given (k, layer list)."""
        seg = B.deft_select(g, self.offsets, k, my_layers, self.idx_out, self.val_out, self.ws)
        kr = int(seg[-1])
        return seg, self.idx_out[:kr], self.val_out[:kr]

    def topk_global(self, g: torch.Tensor, K: Optional[int] = None):
        K = self.K if K is None else int(K)
        B.topk_global(g, K, self.idx_out, self.val_out, self.ws)
        torch.cuda.current_stream().synchronize()
        return self.idx_out[:K].cpu().numpy(), self.val_out[:K].cpu().numpy()
