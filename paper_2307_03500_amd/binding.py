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

DEFT_OK, DEFT_EINVAL, DEFT_ERANGE, DEFT_EWS, DEFT_ECAP, DEFT_EHIP, DEFT_ELIMIT = 0, -1, -2, -3, -4, -5, -6
NOALLOC_MAX_ELEMS = 1 << 30
OP_NORMS, OP_SELECT, OP_TOPK_GLOBAL = 0, 1, 2
SHAPE_AUTO, SHAPE_SHORT, SHAPE_LONG, SHAPE_LONG_PLAIN, SHAPE_LONG_SAMPLED = 0, 1, 2, 3, 4

# Every pointer travels as a plain address (void*): numpy arrays pass `arr.ctypes.data`,
# torch tensors pass `t.data_ptr()`; callers on a hot path cache those integers.
_P = C.c_void_p

SIGNATURES = {
    "deft_strerror": (C.c_char_p, [C.c_int]),
    "deft_partition": (C.c_int, [_P, C.c_int32, C.c_int32, _P, _P, C.c_int32, _P]),
    "deft_check_layout": (C.c_int, [_P, C.c_int32, C.c_int64]),
    "deft_layer_norms": (C.c_int, [_P, C.c_int64, _P, C.c_int32, _P, _P, C.c_size_t, _P]),
    "deft_layer_norms_noalloc": (C.c_int, [_P, C.c_int64, _P, C.c_int32, _P, _P]),
    "deft_norms_from_sumsq": (C.c_int, [_P, C.c_int32, _P]),
    "deft_total_k": (C.c_int, [C.c_int64, C.c_double, _P]),
    "deft_cltk_leader": (C.c_int, [C.c_int64, C.c_int32, _P]),
    "deft_cltk_select": (C.c_int, [_P, C.c_int64, C.c_double, C.c_int32, C.c_int32, C.c_int64, _P, _P,
                                   C.c_int64, _P, C.c_size_t, C.c_int32, _P, _P]),
    "deft_accumulate_norms": (C.c_int, [_P, _P, C.c_float, _P, C.c_int64, _P, C.c_int32, _P, _P,
                                        C.c_size_t, _P]),
    "deft_gather_zero": (C.c_int, [_P, C.c_int64, _P, C.c_int64, _P, _P]),
    "deft_stream_read_probe": (C.c_int, [_P, C.c_int64, _P, _P]),
    "deft_alloc_k": (C.c_int, [_P, _P, C.c_int32, C.c_int64, C.c_double, _P]),
    "deft_assign_layers": (C.c_int, [_P, _P, C.c_int32, C.c_int32, C.c_int64, C.c_int32, _P, _P, _P]),
    "deft_cost_model": (C.c_int, [_P, _P, _P, C.c_int32, C.c_int32, C.c_int64, C.c_int64, _P, _P]),
    "deft_select": (C.c_int, [_P, C.c_int64, _P, _P, C.c_int32, _P, C.c_int32, _P, _P, _P,
                              C.c_int64, _P, C.c_size_t, C.c_int32, _P]),
    "topk_global": (C.c_int, [_P, C.c_int64, C.c_int64, _P, _P, _P, C.c_size_t, C.c_int32, _P]),
    "deft_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int64, C.c_int32]),
    "deft_sparsify": (C.c_int, [_P, _P, C.c_int64, _P, _P, _P, _P]),
    "deft_accumulate_sparsify": (C.c_int, [_P, _P, _P, C.c_float, _P, C.c_int64, _P, _P, _P, _P]),
}

_lib = None


class DeftJob(C.Structure):
    """struct deft_job of deft.h (the per-job arguments of deft_sparsify), field for field."""
    _fields_ = [("N", C.c_int64), ("L", C.c_int32), ("n_workers", C.c_int32), ("rank", C.c_int32),
                ("launch_shape", C.c_int32), ("d", C.c_double), ("offsets_host", _P),
                ("offsets_dev", _P), ("sizes_host", _P), ("sumsq_pinned", _P), ("norms_host", _P),
                ("k_host", _P), ("owner_bin_host", _P), ("my_layers_host", _P),
                ("seg_off_host", _P), ("idx_out_dev", _P), ("val_out_dev", _P),
                ("out_cap", C.c_int64), ("ws_dev", _P), ("ws_bytes", C.c_size_t),
                ("spin_us", C.c_int64)]


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


def _p(a: np.ndarray, typ=None):
    return a.ctypes.data


def _stream(stream) -> int:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


# ---------------------------------------------------------------------------- host calls
def deft_partition(tensor_sizes: Sequence[int], n_workers: int) -> Tuple[np.ndarray, np.ndarray]:
    ts = _i64(tensor_sizes)
    cap = max(1, len(ts) * max(1, int(n_workers)))
    off = np.zeros(cap + 1, np.int64)
    lt = np.zeros(cap, np.int32)
    L = np.zeros(1, np.int32)
    _check(lib().deft_partition(_p(ts), len(ts), int(n_workers), _p(off),
                                _p(lt), cap, _p(L)), "deft_partition")
    return off[:L[0] + 1].copy(), lt[:L[0]].copy()


def deft_check_layout(offsets, N: int) -> int:
    off = _i64(offsets)
    return lib().deft_check_layout(_p(off), len(off) - 1, int(N))


def deft_total_k(N: int, d: float) -> int:
    K = C.c_int64(0)
    _check(lib().deft_total_k(int(N), float(d), C.addressof(K)), "deft_total_k")
    return int(K.value)


def deft_cltk_leader(iteration: int, n_workers: int) -> int:
    leader = C.c_int32(0)
    _check(lib().deft_cltk_leader(int(iteration), int(n_workers), C.addressof(leader)),
           "deft_cltk_leader")
    return int(leader.value)


def deft_norms_from_sumsq(sumsq) -> np.ndarray:
    ss = np.ascontiguousarray(sumsq, dtype=np.float64)
    out = np.zeros_like(ss)
    _check(lib().deft_norms_from_sumsq(_p(ss), len(ss), _p(out)),
           "deft_norms_from_sumsq")
    return out


def deft_alloc_k(norms, sizes, N: int, d: float) -> np.ndarray:
    nr = np.ascontiguousarray(norms, dtype=np.float64)
    sz = _i64(sizes)
    k = np.zeros(len(sz), np.int64)
    _check(lib().deft_alloc_k(_p(nr), _p(sz), len(sz), int(N), float(d),
                              _p(k)), "deft_alloc_k")
    return k


def deft_assign_layers(sizes, k, n_workers: int, iteration: int, rank: int):
    sz, kk = _i64(sizes), _i64(k)
    L = len(sz)
    owner = np.zeros(L, np.int32)
    mine = np.zeros(L, np.int32)
    cnt = np.zeros(1, np.int32)
    _check(lib().deft_assign_layers(_p(sz), _p(kk), L, int(n_workers), int(iteration),
                                    int(rank), _p(owner), _p(mine), _p(cnt)),
           "deft_assign_layers")
    return owner, mine[:cnt[0]].copy()


def deft_cost_model(sizes, k, owner_bin, n_workers: int, N: int, K: int) -> dict:
    sz, kk, ob = _i64(sizes), _i64(k), _i32(owner_bin)
    Ci = np.zeros(int(n_workers), np.float64)
    out = np.zeros(5, np.float64)
    _check(lib().deft_cost_model(_p(sz), _p(kk), _p(ob), len(sz), int(n_workers),
                                 int(N), int(K), _p(Ci), _p(out)), "deft_cost_model")
    return {"C_i": Ci.tolist(), "C_n": out[0], "f_n": out[1], "C_trivial": out[2],
            "f_trivial": out[3], "topk_cost": out[4]}


def deft_workspace_bytes(op: int, elems: int, count: int) -> int:
    return int(lib().deft_workspace_bytes(int(op), int(elems), int(count)))


# ---------------------------------------------------------------------------- device calls
def deft_layer_norms(g, offsets_dev, sumsq, ws, stream=None) -> None:
    """g: float32 cuda tensor; offsets_dev: int64 cuda tensor (L+1); sumsq: float64 tensor (L),
    cuda or pinned host; ws: uint8 cuda tensor.  Enqueues only."""
    L = offsets_dev.numel() - 1
    _check(lib().deft_layer_norms(g.data_ptr(), g.numel(),
                                  offsets_dev.data_ptr(), L,
                                  sumsq.data_ptr(), ws.data_ptr(),
                                  ws.numel() * ws.element_size(), _stream(stream)),
           "deft_layer_norms")


def deft_layer_norms_noalloc(g, offsets_dev, sumsq, stream=None) -> None:
    """deft_layer_norms without a workspace argument (scratch built into the library)."""
    L = offsets_dev.numel() - 1
    _check(lib().deft_layer_norms_noalloc(g.data_ptr(), g.numel(), offsets_dev.data_ptr(), L,
                                          sumsq.data_ptr(), _stream(stream)),
           "deft_layer_norms_noalloc")


def deft_accumulate_norms(e, grad, eta: float, acc, offsets_dev, sumsq, ws, stream=None) -> None:
    """acc = e + eta*grad (fp32) and the per-layer sums of squares of acc, one pass.  acc may be e."""
    L = offsets_dev.numel() - 1
    _check(lib().deft_accumulate_norms(e.data_ptr(), grad.data_ptr(), float(eta), acc.data_ptr(),
                                       e.numel(), offsets_dev.data_ptr(), L, sumsq.data_ptr(),
                                       ws.data_ptr(), ws.numel() * ws.element_size(),
                                       _stream(stream)), "deft_accumulate_norms")


def deft_gather_zero(acc, idx, vals_out, stream=None) -> None:
    """vals_out[i] = acc[idx[i]]; acc[idx[i]] = 0.  idx: int32 cuda tensor of distinct positions."""
    _check(lib().deft_gather_zero(acc.data_ptr(), acc.numel(), idx.data_ptr(), idx.numel(),
                                  vals_out.data_ptr(), _stream(stream)), "deft_gather_zero")


def deft_stream_read_probe(g, out, stream=None) -> None:
    """Measurement aid: one streaming read of g in the norm pass's launch shape."""
    _check(lib().deft_stream_read_probe(g.data_ptr(), g.numel(), out.data_ptr(), _stream(stream)),
           "deft_stream_read_probe")


def deft_select(g, offsets_host, k_host, my_layers_host, idx_out, val_out, ws, stream=None,
                shape: int = SHAPE_AUTO) -> np.ndarray:
    """Enqueues Alg. 5 for the given layers; returns seg_off (host, int64, len my_count+1)."""
    off, kk, mine = _i64(offsets_host), _i64(k_host), _i32(my_layers_host)
    seg = np.zeros(len(mine) + 1, np.int64)
    _check(lib().deft_select(g.data_ptr(), g.numel(), _p(off), _p(kk),
                             len(off) - 1, _p(mine), len(mine),
                             idx_out.data_ptr(), val_out.data_ptr(),
                             _p(seg), idx_out.numel(), ws.data_ptr(),
                             ws.numel() * ws.element_size(), int(shape), _stream(stream)),
           "deft_select")
    return seg


def topk_global(g, K: int, idx_out, val_out, ws, stream=None, shape: int = SHAPE_AUTO) -> None:
    _check(lib().topk_global(g.data_ptr(), g.numel(), int(K),
                             idx_out.data_ptr(), val_out.data_ptr(),
                             ws.data_ptr(), ws.numel() * ws.element_size(), int(shape),
                             _stream(stream)), "topk_global")


def deft_cltk_select(g, d: float, n_workers: int, rank: int, iteration: int, idx_out, val_out, ws,
                     stream=None, shape: int = SHAPE_AUTO) -> int:
    """Cyclic local Top-k: enqueues the conventional Top-k on the iteration's leader only;
    returns the number of entries this rank selected (K or 0)."""
    cnt = C.c_int64(0)
    _check(lib().deft_cltk_select(g.data_ptr(), g.numel(), float(d), int(n_workers), int(rank),
                                  int(iteration), idx_out.data_ptr(), val_out.data_ptr(),
                                  idx_out.numel(), ws.data_ptr(), ws.numel() * ws.element_size(),
                                  int(shape), _stream(stream), C.addressof(cnt)),
           "deft_cltk_select")
    return int(cnt.value)


def deft_sparsify(job: DeftJob, g, iteration: int, stream=None, norms_done_event: int = 0):
    """The whole sparsifier call on g; returns (my_count, k_r).  Blocks until the norm pass has
    delivered its sums; the selection is enqueued when it returns."""
    cnt = C.c_int32(0)
    kr = C.c_int64(0)
    _check(lib().deft_sparsify(C.addressof(job), g.data_ptr(), int(iteration), _stream(stream),
                               int(norms_done_event), C.addressof(cnt), C.addressof(kr)),
           "deft_sparsify")
    return int(cnt.value), int(kr.value)


def deft_accumulate_sparsify(job: DeftJob, e, grad, eta: float, acc, iteration: int, stream=None,
                             norms_done_event: int = 0):
    """acc = e + eta*grad, then the whole sparsifier call on acc; returns (my_count, k_r)."""
    cnt = C.c_int32(0)
    kr = C.c_int64(0)
    _check(lib().deft_accumulate_sparsify(C.addressof(job), e.data_ptr(), grad.data_ptr(),
                                          float(eta), acc.data_ptr(), int(iteration),
                                          _stream(stream), int(norms_done_event),
                                          C.addressof(cnt), C.addressof(kr)),
           "deft_accumulate_sparsify")
    return int(cnt.value), int(kr.value)
