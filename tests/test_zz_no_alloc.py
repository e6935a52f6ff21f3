"""The entry point that allocates nothing (deft_layer_norms_noalloc: partial sums in an array
built into the library) against deft_layer_norms and the oracle, through the C ABI: two calls in
a row on one GPU, the second on a smaller input, so that what the first left in the shared
array would show if it were read."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import deft_oracle as O
from paper_2307_03500_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _norms_both_ways(B, g, off):
    gd = torch.from_numpy(g).to(DEV)
    off_d = torch.from_numpy(np.asarray(off, np.int64)).to(DEV)
    L = len(off) - 1
    ws = torch.empty(B.deft_workspace_bytes(B.OP_NORMS, len(g), L), dtype=torch.uint8, device=DEV)
    a = torch.full((L,), -1.0, dtype=torch.float64, device=DEV)
    b = torch.full((L,), -2.0, dtype=torch.float64, device=DEV)
    B.deft_layer_norms(gd, off_d, a, ws)
    before = torch.cuda.memory_allocated()
    B.deft_layer_norms_noalloc(gd, off_d, b)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy()


def test_noalloc_norms_two_calls_second_smaller(deft):
    B = deft
    big = synth.make("resnet18", seed=3)              # 11.7 M elements, 122 layers
    off_big, _ = B.deft_partition(big.tensor_sizes, big.n_workers)
    a, b = _norms_both_ways(B, big.g, off_big)
    assert (a.view(np.uint64) == b.view(np.uint64)).all()   # same kernels, same order: same bits
    want = O.layer_sumsq(big.g, off_big.tolist())
    assert (np.abs(b - want) <= 1e-12 * want).all()
    # second call, smaller and ragged: chunks that the first call filled are partly rewritten
    rng = np.random.default_rng(12)
    sizes = [1, 63, 4097, 5, 16384, 3, 8190, 40000, 2]
    g = (rng.standard_normal(sum(sizes)) * 10 ** rng.uniform(-3, 2, sum(sizes))).astype(np.float32)
    off = np.concatenate([[0], np.cumsum(sizes)])
    a, b = _norms_both_ways(B, g, off)
    assert (a.view(np.uint64) == b.view(np.uint64)).all()
    want = O.layer_sumsq(g, off.tolist())
    assert (np.abs(b - want) <= 1e-12 * want).all()


def test_noalloc_norms_rejects_what_it_cannot_hold(deft):
    B, lib = deft, deft.lib()
    assert lib.deft_layer_norms_noalloc(C.c_void_p(0x1000), B.NOALLOC_MAX_ELEMS + 1,
                                        C.c_void_p(0x2000), 1, C.c_void_p(0x3000), None) == B.DEFT_ELIMIT
    assert lib.deft_layer_norms_noalloc(C.c_void_p(0x1000), 2 ** 31, C.c_void_p(0x2000), 1,
                                        C.c_void_p(0x3000), None) == B.DEFT_ERANGE
    assert lib.deft_layer_norms_noalloc(None, 16, C.c_void_p(0x2000), 1, C.c_void_p(0x3000),
                                        None) == B.DEFT_EINVAL
    assert "no-allocation" in lib.deft_strerror(B.DEFT_ELIMIT).decode()
