"""Thin ctypes binding over the C ABI declared in include/deft.h.

Argument marshalling only: every step of the path runs inside the library.  Device buffers
are torch tensors (torch is used for device memory and streams, nothing else); host arrays
are numpy.  There is no CPU fallback: if the library is missing, every call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdeft.so")

DEFT_OK, DEFT_EINVAL, DEFT_ERANGE, DEFT_EWS, DEFT_ECAP, DEFT_EHIP = 0, -1, -2, -3, -4, -5
OP_NORMS, OP_SELECT, OP_TOPK_GLOBAL = 0, 1, 2

_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)
_f64p = C.POINTER(C.c_double)

SIGNATURES = {
    "deft_strerror": (C.c_char_p, [C.c_int]),
    "deft_partition": (C.c_int, [_i64p, C.c_int32, C.c_int32, _i64p, _i32p, C.c_int32, _i32p]),
    "deft_check_layout": (C.c_int, [_i64p, C.c_int32, C.c_int64]),
    "deft_layer_norms": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]),
    "deft_norms_from_sumsq": (C.c_int, [_f64p, C.c_int32, _f64p]),
    "deft_alloc_k": (C.c_int, [_f64p, _i64p, C.c_int32, C.c_int64, C.c_double, _i64p]),
    "deft_assign_layers": (C.c_int, [_i64p, _i64p, C.c_int32, C.c_int32, C.c_int64, C.c_int32,
                                     _i32p, _i32p, _i32p]),
    "deft_cost_model": (C.c_int, [_i64p, _i64p, _i32p, C.c_int32, C.c_int32, C.c_int64,
                                  C.c_int64, _f64p, _f64p]),
    "deft_select": (C.c_int, [C.c_void_p, C.c_int64, _i64p, _i64p, C.c_int32, _i32p, C.c_int32,
                              C.c_void_p, C.c_void_p, _i64p, C.c_int64, C.c_void_p, C.c_size_t,
                              C.c_void_p]),
    "topk_global": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_size_t, C.c_void_p]),
    "deft_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int64, C.c_int32]),
}

_lib = None


class DeftError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().deft_strerror(status).decode()} (status {status})")


def lib():
    """Load the in-tree library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; "
                "g.build()'` from the repository root; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != DEFT_OK:
        raise DeftError(status, where)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray, typ):
    return a.ctypes.data_as(typ)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(int(stream.cuda_stream))


# ---------------------------------------------------------------------------- host calls
def deft_partition(tensor_sizes: Sequence[int], n_workers: int) -> Tuple[np.ndarray, np.ndarray]:
    ts = _i64(tensor_sizes)
    cap = max(1, len(ts) * max(1, int(n_workers)))
    off = np.zeros(cap + 1, np.int64)
    lt = np.zeros(cap, np.int32)
    L = C.c_int32(0)
    _check(lib().deft_partition(_p(ts, _i64p), len(ts), int(n_workers), _p(off, _i64p),
                                _p(lt, _i32p), cap, C.byref(L)), "deft_partition")
    return off[:L.value + 1].copy(), lt[:L.value].copy()


def deft_check_layout(offsets, N: int) -> int:
    off = _i64(offsets)
    return lib().deft_check_layout(_p(off, _i64p), len(off) - 1, int(N))


def deft_norms_from_sumsq(sumsq) -> np.ndarray:
    ss = np.ascontiguousarray(sumsq, dtype=np.float64)
    out = np.zeros_like(ss)
    _check(lib().deft_norms_from_sumsq(_p(ss, _f64p), len(ss), _p(out, _f64p)),
           "deft_norms_from_sumsq")
    return out


def deft_alloc_k(norms, sizes, N: int, d: float) -> np.ndarray:
    nr = np.ascontiguousarray(norms, dtype=np.float64)
    sz = _i64(sizes)
    k = np.zeros(len(sz), np.int64)
    _check(lib().deft_alloc_k(_p(nr, _f64p), _p(sz, _i64p), len(sz), int(N), float(d),
                              _p(k, _i64p)), "deft_alloc_k")
    return k


def deft_assign_layers(sizes, k, n_workers: int, iteration: int, rank: int):
    sz, kk = _i64(sizes), _i64(k)
    L = len(sz)
    owner = np.zeros(L, np.int32)
    mine = np.zeros(L, np.int32)
    cnt = C.c_int32(0)
    _check(lib().deft_assign_layers(_p(sz, _i64p), _p(kk, _i64p), L, int(n_workers), int(iteration),
                                    int(rank), _p(owner, _i32p), _p(mine, _i32p), C.byref(cnt)),
           "deft_assign_layers")
    return owner, mine[:cnt.value].copy()


def deft_cost_model(sizes, k, owner_bin, n_workers: int, N: int, K: int) -> dict:
    sz, kk, ob = _i64(sizes), _i64(k), _i32(owner_bin)
    Ci = np.zeros(int(n_workers), np.float64)
    out = np.zeros(5, np.float64)
    _check(lib().deft_cost_model(_p(sz, _i64p), _p(kk, _i64p), _p(ob, _i32p), len(sz), int(n_workers),
                                 int(N), int(K), _p(Ci, _f64p), _p(out, _f64p)), "deft_cost_model")
    return {"C_i": Ci.tolist(), "C_n": out[0], "f_n": out[1], "C_trivial": out[2],
            "f_trivial": out[3], "topk_cost": out[4]}


def deft_workspace_bytes(op: int, elems: int, count: int) -> int:
    return int(lib().deft_workspace_bytes(int(op), int(elems), int(count)))


# ---------------------------------------------------------------------------- device calls
def deft_layer_norms(g, offsets_dev, sumsq, ws, stream=None) -> None:
    """g: float32 cuda tensor; offsets_dev: int64 cuda tensor (L+1); sumsq: float64 tensor (L),
    cuda or pinned host; ws: uint8 cuda tensor.  Enqueues only."""
    L = offsets_dev.numel() - 1
    _check(lib().deft_layer_norms(C.c_void_p(g.data_ptr()), g.numel(),
                                  C.c_void_p(offsets_dev.data_ptr()), L,
                                  C.c_void_p(sumsq.data_ptr()), C.c_void_p(ws.data_ptr()),
                                  ws.numel() * ws.element_size(), _stream(stream)),
           "deft_layer_norms")


def deft_select(g, offsets_host, k_host, my_layers_host, idx_out, val_out, ws, stream=None) -> np.ndarray:
    """Enqueues Alg. 5 for the given layers; returns seg_off (host, int64, len my_count+1)."""
    off, kk, mine = _i64(offsets_host), _i64(k_host), _i32(my_layers_host)
    seg = np.zeros(len(mine) + 1, np.int64)
    _check(lib().deft_select(C.c_void_p(g.data_ptr()), g.numel(), _p(off, _i64p), _p(kk, _i64p),
                             len(off) - 1, _p(mine, _i32p), len(mine),
                             C.c_void_p(idx_out.data_ptr()), C.c_void_p(val_out.data_ptr()),
                             _p(seg, _i64p), idx_out.numel(), C.c_void_p(ws.data_ptr()),
                             ws.numel() * ws.element_size(), _stream(stream)), "deft_select")
    return seg


def topk_global(g, K: int, idx_out, val_out, ws, stream=None) -> None:
    _check(lib().topk_global(C.c_void_p(g.data_ptr()), g.numel(), int(K),
                             C.c_void_p(idx_out.data_ptr()), C.c_void_p(val_out.data_ptr()),
                             C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size(),
                             _stream(stream)), "topk_global")
