"""One worker's DEFT sparsifier (Sec. 4 of the paper) as a sequence of C-ABI calls.

This class only owns buffers and orders the calls; it computes nothing itself:
  deft_partition (once) -> deft_layer_norms [device] -> stream sync ->
  deft_norms_from_sumsq -> deft_alloc_k -> deft_assign_layers [host] -> deft_select [device].
torch supplies device memory, pinned host memory and the stream.  All host arrays are
allocated once and their addresses cached, so a call costs a few ctypes invocations.
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
    idx_dev: torch.Tensor   # int32 [k_r] global indices, device (view of the selector's buffer)
    val_dev: torch.Tensor   # float32 [k_r] values, device (view of the selector's buffer)
    times: dict = field(default_factory=dict)

    @property
    def idx(self) -> np.ndarray:
        return self.idx_dev.cpu().numpy()

    @property
    def val(self) -> np.ndarray:
        return self.val_dev.cpu().numpy()


# Launch shape of selectors that are not given one (tests switch it to run the long-vector
# kernels on small inputs; it changes speed only).
DEFAULT_SHAPE = B.SHAPE_AUTO


class DeftSelector:
    def __init__(self, tensor_sizes: Sequence[int], n_workers: int, d: float, device,
                 out_cap: Optional[int] = None, shape: Optional[int] = None, spin_us: int = 0):
        self.device = torch.device(device)
        self.n = int(n_workers)
        self.d = float(d)
        # launch shape handed to every selection call
        self.shape = DEFAULT_SHAPE if shape is None else int(shape)
        self.spin_us = int(spin_us)  # deft_job.spin_us
        self.offsets, self.layer_tensor = B.deft_partition(tensor_sizes, n_workers)
        self.L = L = len(self.offsets) - 1
        self.N = int(self.offsets[-1])
        self.sizes = np.diff(self.offsets).astype(np.int64)
        self.K = B.deft_total_k(self.N, self.d)
        dev = self.device
        self.offsets_dev = torch.from_numpy(self.offsets).to(dev)
        self.sumsq_host = torch.zeros(L, dtype=torch.float64).pin_memory()
        nb = max(B.deft_workspace_bytes(B.OP_NORMS, self.N, L),
                 B.deft_workspace_bytes(B.OP_SELECT, self.N, L),
                 B.deft_workspace_bytes(B.OP_TOPK_GLOBAL, self.N, 1))
        self.ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        # sum of k_l can exceed K by the number of layers clamped up to 1 (Alg. 3)
        self.out_cap = int(out_cap) if out_cap is not None else self.K + L + 1
        cap = max(self.out_cap, self.K, 1)
        self.idx_out = torch.empty(cap, dtype=torch.int32, device=dev)
        self.val_out = torch.empty(cap, dtype=torch.float32, device=dev)
        # persistent host arrays of the plan
        self.norms_h = np.zeros(L, np.float64)
        self.k_h = np.zeros(L, np.int64)
        self.owner_h = np.zeros(L, np.int32)
        self.mine_h = np.zeros(L, np.int32)
        self.cnt_h = np.zeros(1, np.int32)
        self.seg_h = np.zeros(L + 1, np.int64)
        # cached addresses
        self._lib = B.lib()
        self._p = {
            "off_dev": self.offsets_dev.data_ptr(), "sumsq": self.sumsq_host.data_ptr(),
            "ws": self.ws.data_ptr(), "ws_bytes": nb, "idx": self.idx_out.data_ptr(),
            "val": self.val_out.data_ptr(), "off": self.offsets.ctypes.data,
            "sizes": self.sizes.ctypes.data, "norms": self.norms_h.ctypes.data,
            "k": self.k_h.ctypes.data, "owner": self.owner_h.ctypes.data,
            "mine": self.mine_h.ctypes.data, "cnt": self.cnt_h.ctypes.data,
            "seg": self.seg_h.ctypes.data,
        }
        self._cap = cap
        self._jobs = {}
        self._cnt_c = B.C.c_int32(0)
        self._kr_c = B.C.c_int64(0)
        self._cnt_p, self._kr_p = B.C.addressof(self._cnt_c), B.C.addressof(self._kr_c)

    def _job(self, rank: int) -> int:
        """Address of this rank's deft_job (built once, kept alive by the selector)."""
        j = self._jobs.get(rank)
        if j is None:
            p = self._p
            j = B.DeftJob(self.N, self.L, self.n, int(rank), self.shape, self.d, p["off"],
                          p["off_dev"], p["sizes"], p["sumsq"], p["norms"], p["k"], p["owner"],
                          p["mine"], p["seg"], p["idx"], p["val"], self._cap, p["ws"],
                          p["ws_bytes"], self.spin_us)
            self._jobs[rank] = j
        return B.C.addressof(j)

    # -- steps (each is one or a few C-ABI calls on cached addresses) ----------------------
    def enqueue_norms(self, g: torch.Tensor, stream_handle: int) -> None:
        p = self._p
        rc = self._lib.deft_layer_norms(g.data_ptr(), self.N, p["off_dev"], self.L, p["sumsq"],
                                        p["ws"], p["ws_bytes"], stream_handle)
        if rc:
            raise B.DeftError(rc, "deft_layer_norms")

    def plan_host(self, rank: int, iteration: int) -> int:
        """sumsq (already on the host) -> norms -> k -> bins; returns this rank's layer count."""
        p, lib, L = self._p, self._lib, self.L
        rc = lib.deft_norms_from_sumsq(p["sumsq"], L, p["norms"])
        if rc:
            raise B.DeftError(rc, "deft_norms_from_sumsq")
        rc = lib.deft_alloc_k(p["norms"], p["sizes"], L, self.N, self.d, p["k"])
        if rc:
            raise B.DeftError(rc, "deft_alloc_k")
        rc = lib.deft_assign_layers(p["sizes"], p["k"], L, self.n, iteration, rank, p["owner"],
                                    p["mine"], p["cnt"])
        if rc:
            raise B.DeftError(rc, "deft_assign_layers")
        return int(self.cnt_h[0])

    def enqueue_select(self, g: torch.Tensor, count: int, stream_handle: int) -> int:
        """Alg. 5 on the planned layers; returns k_r."""
        p = self._p
        rc = self._lib.deft_select(g.data_ptr(), self.N, p["off"], p["k"], self.L, p["mine"], count,
                                   p["idx"], p["val"], p["seg"], self._cap, p["ws"], p["ws_bytes"],
                                   self.shape, stream_handle)
        if rc:
            raise B.DeftError(rc, "deft_select")
        return int(self.seg_h[count])

    # -- convenience wrappers ---------------------------------------------------------------
    def norms(self, g: torch.Tensor) -> np.ndarray:
        st = torch.cuda.current_stream()
        self.enqueue_norms(g, st.cuda_stream)
        st.synchronize()
        return B.deft_norms_from_sumsq(self.sumsq_host.numpy())

    def select(self, g: torch.Tensor, rank: int, iteration: int = 0) -> Selection:
        assert g.dtype == torch.float32 and g.numel() == self.N and g.device == self.device
        st = torch.cuda.current_stream()
        h = st.cuda_stream
        t0 = time.perf_counter()
        self.enqueue_norms(g, h)
        st.synchronize()
        t1 = time.perf_counter()
        cnt = self.plan_host(rank, iteration)
        t2 = time.perf_counter()
        kr = self.enqueue_select(g, cnt, h)
        st.synchronize()
        t3 = time.perf_counter()
        return Selection(self.norms_h.copy(), self.k_h.copy(), self.owner_h.copy(),
                         self.mine_h[:cnt].copy(), self.seg_h[:cnt + 1].copy(),
                         self.idx_out[:kr], self.val_out[:kr],
                         {"norm_ms": (t1 - t0) * 1e3, "plan_ms": (t2 - t1) * 1e3,
                          "select_ms": (t3 - t2) * 1e3})

    def enqueue_sparsify(self, g: torch.Tensor, rank: int, iteration: int, stream_handle: int,
                         norms_done_event: int = 0):
        """deft_sparsify: the whole call in one library entry; returns (my_count, k_r) with the
        selection enqueued (not yet complete) on the stream."""
        rc = self._lib.deft_sparsify(self._job(rank), g.data_ptr(), iteration, stream_handle,
                                     norms_done_event, self._cnt_p, self._kr_p)
        if rc:
            raise B.DeftError(rc, "deft_sparsify")
        return self._cnt_c.value, self._kr_c.value

    def sparsify(self, g: torch.Tensor, rank: int, iteration: int = 0) -> Selection:
        """Same result as select(), through the single entry point."""
        assert g.dtype == torch.float32 and g.numel() == self.N and g.device == self.device
        st = torch.cuda.current_stream()
        t0 = time.perf_counter()
        cnt, kr = self.enqueue_sparsify(g, rank, iteration, st.cuda_stream)
        st.synchronize()
        t1 = time.perf_counter()
        return Selection(self.norms_h.copy(), self.k_h.copy(), self.owner_h.copy(),
                         self.mine_h[:cnt].copy(), self.seg_h[:cnt + 1].copy(),
                         self.idx_out[:kr], self.val_out[:kr], {"step_ms": (t1 - t0) * 1e3})

    def accumulate_sparsify(self, e: torch.Tensor, grad: torch.Tensor, eta: float,
                            acc: torch.Tensor, rank: int, iteration: int = 0) -> Selection:
        """Alg. 1's accumulation and the sparsifier call on its result, one library entry."""
        for t in (e, grad, acc):
            assert t.dtype == torch.float32 and t.numel() == self.N and t.device == self.device
        st = torch.cuda.current_stream()
        rc = self._lib.deft_accumulate_sparsify(self._job(rank), e.data_ptr(), grad.data_ptr(),
                                                float(eta), acc.data_ptr(), iteration,
                                                st.cuda_stream, 0, self._cnt_p, self._kr_p)
        if rc:
            raise B.DeftError(rc, "deft_accumulate_sparsify")
        st.synchronize()
        cnt, kr = self._cnt_c.value, self._kr_c.value
        return Selection(self.norms_h.copy(), self.k_h.copy(), self.owner_h.copy(),
                         self.mine_h[:cnt].copy(), self.seg_h[:cnt + 1].copy(),
                         self.idx_out[:kr], self.val_out[:kr])

    def select_with_plan(self, g: torch.Tensor, k: np.ndarray, my_layers: np.ndarray):
        """Alg. 5 alone, for a given (k, layer list)."""
        seg = B.deft_select(g, self.offsets, k, my_layers, self.idx_out, self.val_out, self.ws,
                            shape=self.shape)
        kr = int(seg[-1])
        return seg, self.idx_out[:kr], self.val_out[:kr]

    def topk_global(self, g: torch.Tensor, K: Optional[int] = None):
        K = self.K if K is None else int(K)
        B.topk_global(g, K, self.idx_out, self.val_out, self.ws, shape=self.shape)
        torch.cuda.current_stream().synchronize()
        return self.idx_out[:K].cpu().numpy(), self.val_out[:K].cpu().numpy()

    def cltk(self, g: torch.Tensor, rank: int, iteration: int):
        """Cyclic local Top-k (the comparison scheme of Sec. 1 / Sec. 3.1): the worker whose rank
        equals iteration % n selects the conventional Top-k of its whole vector (to be broadcast
        by the caller); every other worker selects nothing and waits.  Returns (idx, val) or None."""
        cnt = B.deft_cltk_select(g, self.d, self.n, rank, iteration, self.idx_out, self.val_out,
                                 self.ws, shape=self.shape)
        if cnt == 0:
            return None
        torch.cuda.current_stream().synchronize()
        return self.idx_out[:cnt].cpu().numpy(), self.val_out[:cnt].cpu().numpy()
