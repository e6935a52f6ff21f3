"""Randomised GPU parity: many seeded shapes, value kinds, k choices and layer subsets, in both
launch shapes of the selection, each compared element by element with the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import deft_oracle as O
from paper_2307_03500_amd import binding as B
from paper_2307_03500_amd import pipeline

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _values(rng, N, kind):
    if kind == 0:
        g = rng.standard_normal(N)
    elif kind == 1:
        g = rng.standard_t(3.0, N) * 10 ** rng.uniform(-4, 1)
    elif kind == 2:  # few distinct magnitudes, both signs, many zeros
        g = rng.integers(-5, 6, N) * 0.125
        g[rng.random(N) < 0.5] = 0.0
    elif kind == 3:  # rounded through bf16: at most 15 varying key bits
        g = rng.standard_t(3.0, N).astype(np.float32)
        u = g.view(np.uint32)
        u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        u &= np.uint32(0xFFFF0000)
        return g
    elif kind == 4:  # blocks of rows that are entirely zero, like unused embedding rows
        g = rng.laplace(0, 1e-2, N)
        row = 37
        rows = N // row
        dead = rng.random(rows) < 0.8
        g[:rows * row].reshape(rows, row)[dead] = 0.0
    else:  # per-position scale drifting over 6 decades: only a few chunks hold the large keys
        g = rng.standard_normal(N) * 10 ** np.linspace(-6, 0, N)
    return g.astype(np.float32)


@pytest.mark.parametrize("seed", range(48))
def test_random_layers_and_k(deft, seed):
    rng = np.random.default_rng(7000 + seed)
    long_shape = seed % 3 == 2
    shape = (B.SHAPE_LONG_SAMPLED if seed % 2 else B.SHAPE_LONG_PLAIN) if long_shape else B.SHAPE_AUTO
    try:
        n_layers = int(rng.integers(1, 40))
        top = int(10 ** rng.uniform(1, 5.6))
        sizes = [int(x) for x in rng.integers(1, top + 1, n_layers)]
        N = sum(sizes)
        g = _values(rng, N, seed % 6)
        sel = pipeline.DeftSelector(sizes, 1, 0.5, DEV, out_cap=N, shape=shape)
        gd = torch.from_numpy(g).to(DEV)
        off = sel.offsets.tolist()
        for trial in range(3):
            mode = (seed + trial) % 4
            if mode == 0:
                k = [int(rng.integers(0, s + 1)) for s in sizes]
            elif mode == 1:
                k = [max(1, int(s * 10 ** rng.uniform(-3, -1))) for s in sizes]
            elif mode == 2:
                k = [min(s, 1 + int(rng.integers(0, 4))) for s in sizes]
            else:
                k = [s - int(rng.integers(0, min(s, 3))) for s in sizes]
            part = list(rng.permutation(n_layers)[:int(rng.integers(1, n_layers + 1))])
            seg, idx_dev, val_dev = sel.select_with_plan(gd, np.asarray(k, np.int64),
                                                         np.asarray(part, np.int32))
            torch.cuda.synchronize()
            o_idx, o_val, o_seg = O.select(g, off, k, part)
            assert seg.tolist() == o_seg.tolist()
            assert idx_dev.cpu().numpy().tolist() == o_idx.tolist()
            assert (val_dev.cpu().numpy().view(np.uint32) == o_val.view(np.uint32)).all()
        # the conventional Top-k over the same vector
        K = int(rng.integers(0, N + 1)) if seed % 2 else max(1, N // 500)
        gi, gv = sel.topk_global(gd, K)
        oi, ov = O.topk_global(g, K)
        assert gi.tolist() == oi.tolist() and (gv.view(np.uint32) == ov.view(np.uint32)).all()
        # norms on the same ragged layout
        got = sel.norms(gd)
        want = O.layer_norms(g, off)
        nz = want > 0
        assert (got[~nz] == 0).all()
        assert (np.abs(got[nz] - want[nz]) / want[nz]).max(initial=0.0) <= 1e-13
    finally:
        pass


@pytest.mark.parametrize("seed", range(16))
def test_random_whole_call(deft, seed):
    """deft_sparsify on random layer lists (fewer and more segments than one descriptor batch
    holds, both launch shapes) against the oracle's whole path fed the GPU's norms."""
    rng = np.random.default_rng(9000 + seed)
    shape = (B.SHAPE_LONG_SAMPLED if seed % 8 == 3 else B.SHAPE_LONG_PLAIN) if seed % 4 == 3 else B.SHAPE_AUTO
    try:
        n_tensors = int(rng.integers(1, 60)) if seed % 2 else int(rng.integers(150, 260))
        top = int(10 ** rng.uniform(1, 4.8))
        sizes = [int(x) for x in rng.integers(1, top + 1, n_tensors)]
        n = int(rng.integers(1, 5))
        d = float(10 ** rng.uniform(-3, -0.5))
        sel = pipeline.DeftSelector(sizes, n, d, DEV, shape=shape)
        N = sel.N
        g = _values(rng, N, seed % 6)
        pos = 0
        for sz in sizes:  # per-tensor scales, so that the norms differ
            g[pos:pos + sz] *= np.float32(10 ** rng.uniform(-3, 0))
            pos += sz
        gd = torch.from_numpy(g).to(DEV)
        off, lay = sel.offsets.tolist(), sel.sizes.tolist()
        for it in range(n):
            r = int(rng.integers(0, n))
            res = sel.sparsify(gd, rank=r, iteration=it)
            k = O.alloc_k(res.norms, lay, N, d)
            assert res.k.tolist() == k
            owner, part, _ = O.assign_layers(lay, k, n, it, r)
            assert res.owner_bin.tolist() == owner and res.my_layers.tolist() == part
            o_idx, o_val, o_seg = O.select(g, off, k, part)
            assert res.seg_off.tolist() == o_seg.tolist()
            assert res.idx.tolist() == o_idx.tolist()
            assert (res.val.view(np.uint32) == o_val.view(np.uint32)).all()
    finally:
        pass
