"""CPU-only tests of the C-ABI library: exported symbols, host planner (Alg. 2, 3, 4, Eq. 3-8)
bit-exact against the oracle, and argument validation.  No compute call touches a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import deft_oracle as O
from paper_2307_03500_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol(deft):
    hdr = open(os.path.join(ROOT, "include", "deft.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b([a-z_0-9]+)\s*\(", hdr)) - {"defined"}
    assert {"deft_layer_norms", "deft_alloc_k", "deft_assign_layers", "deft_select",
            "topk_global", "deft_partition"} <= declared
    L = C.CDLL(deft.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(deft.SIGNATURES)


def test_header_is_plain_c_and_library_links_from_c(deft, tmp_path):
    """include/deft.h compiles as strict C99 and a C program can call the library directly."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "c_abi_check")
    libdir = os.path.dirname(deft.LIB_PATH)
    subprocess.run([cc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi_check.c"),
                    "-L", libdir, "-l:libdeft.so", "-Wl,-rpath," + libdir, "-o", exe], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True)
    assert "c abi ok" in out.stdout


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_partition_matches_oracle_on_configs(deft, name):
    sizes = synth.tensor_sizes(name)
    n = synth.CONFIGS[name].n_workers
    off, lt = deft.deft_partition(sizes, n)
    o_off, o_lt = O.partition(sizes, n)
    assert off.tolist() == o_off and lt.tolist() == o_lt
    assert deft.deft_check_layout(off, sum(sizes)) == 0


@pytest.mark.parametrize("seed", range(40))
def test_partition_matches_oracle_random(deft, seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 30))
    sizes = [int(x) for x in rng.integers(0, 10 ** int(rng.integers(1, 6)), T)]
    if sum(sizes) == 0:
        sizes[0] = 3
    n = int(rng.integers(1, 40))
    off, lt = deft.deft_partition(sizes, n)
    o_off, o_lt = O.partition(sizes, n)
    assert off.tolist() == o_off and lt.tolist() == o_lt


@pytest.mark.parametrize("seed", range(60))
def test_alloc_and_assign_match_oracle_random(deft, seed):
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 400))
    sizes = [int(x) for x in 10 ** rng.uniform(0, 6.5, L)]
    N = sum(sizes)
    norms = 10 ** rng.uniform(-8, 2, L)
    if seed % 4 == 0:
        norms[rng.integers(0, L, max(1, L // 5))] = 0.0
    if seed % 5 == 0:
        norms[:] = norms[0]  # all equal: pure tie-breaking
    d = float(10 ** rng.uniform(-4, 0))
    k = deft.deft_alloc_k(norms, sizes, N, d)
    assert k.tolist() == O.alloc_k(norms, sizes, N, d)
    n = int(rng.integers(1, 40))
    it = int(rng.integers(0, 1000))
    for rank in {0, n - 1, int(rng.integers(0, n))}:
        owner, mine = deft.deft_assign_layers(sizes, k, n, it, rank)
        o_owner, o_part, o_bins = O.assign_layers(sizes, k.tolist(), n, it, rank)
        assert owner.tolist() == o_owner and mine.tolist() == o_part
    cm = deft.deft_cost_model(sizes, k, owner, n, N, max(1, O.total_k(N, d)))
    om = O.cost_model(sizes, k.tolist(), o_bins, N, max(1, O.total_k(N, d)))
    assert cm["C_n"] == pytest.approx(om["C_n"], rel=1e-12)
    assert cm["f_trivial"] == pytest.approx(om["f_trivial"], rel=1e-12)
    assert np.allclose(cm["C_i"], om["C_i"], rtol=1e-12)


def test_equal_costs_tie_breaking(deft):
    # identical layers with identical k: equal non-zero costs everywhere
    sizes = [1000] * 24 + [10] * 7
    k = [50] * 24 + [1] * 7
    for n in (1, 3, 8, 24, 40):
        owner, mine = deft.deft_assign_layers(sizes, k, n, 5, n // 2)
        o_owner, o_part, _ = O.assign_layers(sizes, k, n, 5, n // 2)
        assert owner.tolist() == o_owner and mine.tolist() == o_part


@pytest.mark.parametrize("name", ["toy_mlp", "resnet18", "lstm_lm", "ncf"])
def test_planner_on_config_gradients(deft, name):
    """Whole host plan on a real-shaped gradient set, norms from the oracle."""
    gs = synth.make(name, seed=0)
    off, _ = deft.deft_partition(gs.tensor_sizes, gs.n_workers)
    sizes = np.diff(off)
    norms = O.layer_norms(gs.g, off.tolist())
    assert deft.deft_norms_from_sumsq(O.layer_sumsq(gs.g, off.tolist())).tolist() == norms.tolist()
    k = deft.deft_alloc_k(norms, sizes, gs.N, gs.d)
    assert k.tolist() == O.alloc_k(norms, sizes.tolist(), gs.N, gs.d)
    K = O.total_k(gs.N, gs.d)
    # sum k_l = K + (k_last - rho)   (identity of Alg. 3; equality with K only without clamps)
    order = sorted(range(len(k)), key=lambda l: (-norms[l], l))
    rho = K - int(sum(k[l] for l in order[:-1]))
    assert int(k.sum()) == K + (int(k[order[-1]]) - rho)
    seen = []
    for r in range(gs.n_workers):
        owner, mine = deft.deft_assign_layers(sizes, k, gs.n_workers, 0, r)
        assert mine.tolist() == O.assign_layers(sizes.tolist(), k.tolist(), gs.n_workers, 0, r)[1]
        assert (owner[mine] == r).all()
        seen += mine.tolist()
    assert sorted(seen) == list(range(len(k)))
    cm = deft.deft_cost_model(sizes, k, owner, gs.n_workers, gs.N, K)
    assert cm["f_n"] >= gs.n_workers  # Eq. 9's right-hand bound holds on these sets (no theorem)


def test_host_argument_validation(deft):
    B = deft
    with pytest.raises(B.DeftError) as e:
        B.deft_partition([4, -1], 2)
    assert e.value.status == B.DEFT_EINVAL
    with pytest.raises(B.DeftError) as e:
        B.deft_partition([2 ** 31], 2)
    assert e.value.status == B.DEFT_ERANGE
    with pytest.raises(B.DeftError):
        B.deft_partition([4], 0)
    assert B.deft_check_layout([0, 4, 3, 8], 8) == B.DEFT_EINVAL
    assert B.deft_check_layout([1, 4, 8], 8) == B.DEFT_EINVAL
    assert B.deft_check_layout([0, 4, 8], 9) == B.DEFT_EINVAL
    assert B.deft_check_layout([0, 2 ** 31], 2 ** 31) == B.DEFT_ERANGE
    assert B.deft_check_layout([0, 4, 4, 8], 8) == B.DEFT_OK
    for bad_d in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(B.DeftError):
            B.deft_alloc_k([1.0], [10], 10, bad_d)
    with pytest.raises(B.DeftError):
        B.deft_alloc_k([float("nan")], [10], 10, 0.1)
    with pytest.raises(B.DeftError):
        B.deft_alloc_k([-1.0], [10], 10, 0.1)
    with pytest.raises(B.DeftError):
        B.deft_alloc_k([1.0], [0], 10, 0.1)
    with pytest.raises(B.DeftError):
        B.deft_assign_layers([10], [1], 0, 0, 0)
    with pytest.raises(B.DeftError):
        B.deft_assign_layers([10], [1], 4, 0, 4)
    with pytest.raises(B.DeftError):
        B.deft_assign_layers([10], [11], 4, 0, 0)
    with pytest.raises(B.DeftError):
        B.deft_assign_layers([10], [1], 4, -1, 0)
    with pytest.raises(B.DeftError):
        B.deft_norms_from_sumsq([-1.0])
    assert B.deft_workspace_bytes(99, 10, 1) == 0
    assert B.deft_workspace_bytes(B.OP_SELECT, -1, 1) == 0
    assert B.deft_workspace_bytes(B.OP_NORMS, 10 ** 6, 5) >= 2 * 8 * (10 ** 6 // 8192)
    assert B.lib().deft_strerror(B.DEFT_EWS).decode() == "workspace too small"


def test_device_calls_reject_bad_arguments_before_touching_the_gpu(deft):
    """Validation errors are returned before anything is enqueued, so these run without a GPU."""
    B, lib = deft, deft.lib()
    off = np.array([0, 8, 16], np.int64)
    k = np.array([2, 2], np.int64)
    mine = np.array([0, 1], np.int32)
    seg = np.zeros(3, np.int64)
    i64p, i32p = C.POINTER(C.c_int64), C.POINTER(C.c_int32)

    def sel(g=0x1000, N=16, offp=off, kk=k, my=mine, cnt=2, idx=0x2000, val=0x3000, cap=16,
            ws=0x4000, wsb=1 << 20, shape=B.SHAPE_AUTO):
        return lib.deft_select(C.c_void_p(g), N, offp.ctypes.data_as(i64p), kk.ctypes.data_as(i64p),
                               len(offp) - 1, my.ctypes.data_as(i32p), cnt, C.c_void_p(idx),
                               C.c_void_p(val), seg.ctypes.data_as(i64p), cap, C.c_void_p(ws), wsb,
                               shape, None)

    assert sel(shape=5) == B.DEFT_EINVAL and sel(shape=-1) == B.DEFT_EINVAL
    assert sel(g=0) == B.DEFT_EINVAL
    assert sel(g=0x1004) == B.DEFT_EINVAL                      # misaligned vector
    assert sel(N=17) == B.DEFT_EINVAL                          # offsets[L] != N
    assert sel(kk=np.array([2, 9], np.int64)) == B.DEFT_EINVAL  # k > size
    assert sel(my=np.array([0, 2], np.int32)) == B.DEFT_EINVAL  # layer id out of range
    assert sel(cap=3) == B.DEFT_ECAP
    assert sel(wsb=16) == B.DEFT_EWS
    assert sel(cnt=-1) == B.DEFT_EINVAL
    assert sel(cnt=0) == B.DEFT_OK and seg[0] == 0              # nothing to do, nothing enqueued
    assert sel(kk=np.array([0, 0], np.int64)) == B.DEFT_OK      # all k = 0: nothing enqueued

    def norms(g=0x1000, N=16, offd=0x5000, L=2, out=0x6000, ws=0x4000, wsb=1 << 20):
        return lib.deft_layer_norms(C.c_void_p(g), N, C.c_void_p(offd), L, C.c_void_p(out),
                                    C.c_void_p(ws), wsb, None)

    assert norms(g=0) == B.DEFT_EINVAL
    assert norms(L=0) == B.DEFT_EINVAL
    assert norms(N=2 ** 31) == B.DEFT_ERANGE
    assert norms(wsb=8) == B.DEFT_EWS
    assert norms(g=0x1008) == B.DEFT_EINVAL

    def accn(e=0x1000, gr=0x7000, acc=0x1000, N=16, offd=0x5000, L=2, out=0x6000, ws=0x4000, wsb=1 << 20):
        return lib.deft_accumulate_norms(C.c_void_p(e), C.c_void_p(gr), 0.1, C.c_void_p(acc), N,
                                         C.c_void_p(offd), L, C.c_void_p(out), C.c_void_p(ws), wsb, None)

    assert accn(gr=0) == B.DEFT_EINVAL
    assert accn(acc=0) == B.DEFT_EINVAL
    assert accn(acc=0x1004) == B.DEFT_EINVAL
    assert accn(e=0) == B.DEFT_EINVAL
    assert accn(N=2 ** 31) == B.DEFT_ERANGE
    assert accn(wsb=8) == B.DEFT_EWS

    def gz(acc=0x1000, N=16, idx=0x2000, count=4, vals=0x3000):
        return lib.deft_gather_zero(C.c_void_p(acc), N, C.c_void_p(idx), count, C.c_void_p(vals), None)

    assert gz(count=-1) == B.DEFT_EINVAL
    assert gz(acc=0) == B.DEFT_EINVAL
    assert gz(idx=0) == B.DEFT_EINVAL
    assert gz(N=0) == B.DEFT_EINVAL
    assert gz(N=2 ** 31) == B.DEFT_ERANGE
    assert gz(count=0, acc=0, idx=0, vals=0) == B.DEFT_OK

    # deft_sparsify: every refusal comes before the first write to the caller's arrays
    sizes = np.diff(off).astype(np.int64)
    bufs = {"norms": np.zeros(2), "k": np.zeros(2, np.int64), "owner": np.zeros(2, np.int32),
            "mine": np.zeros(2, np.int32), "seg": np.zeros(3, np.int64)}
    cnt, kr = C.c_int32(-7), C.c_int64(-7)

    def spars(g=0x1000, **over):
        f = dict(N=16, L=2, n_workers=2, rank=0, launch_shape=0, d=0.25, offsets_host=off.ctypes.data,
                 offsets_dev=0x5000, sizes_host=sizes.ctypes.data, sumsq_pinned=0x6000,
                 norms_host=bufs["norms"].ctypes.data, k_host=bufs["k"].ctypes.data,
                 owner_bin_host=bufs["owner"].ctypes.data, my_layers_host=bufs["mine"].ctypes.data,
                 seg_off_host=bufs["seg"].ctypes.data, idx_out_dev=0x2000, val_out_dev=0x3000,
                 out_cap=16, ws_dev=0x4000, ws_bytes=1 << 20)
        f.update(over)
        job = B.DeftJob(**f)
        return lib.deft_sparsify(C.addressof(job), C.c_void_p(g), 0, None, None,
                                 C.addressof(cnt), C.addressof(kr))

    assert lib.deft_sparsify(None, C.c_void_p(0x1000), 0, None, None, C.addressof(cnt),
                             C.addressof(kr)) == B.DEFT_EINVAL
    assert spars(g=0) == B.DEFT_EINVAL
    assert spars(g=0x1004) == B.DEFT_EINVAL
    assert spars(rank=2) == B.DEFT_EINVAL
    assert spars(launch_shape=7) == B.DEFT_EINVAL
    assert spars(n_workers=0) == B.DEFT_EINVAL
    assert spars(d=0.0) == B.DEFT_EINVAL
    assert spars(d=1.5) == B.DEFT_EINVAL
    assert spars(N=17) == B.DEFT_EINVAL
    wrong_sizes = np.array([8, 7], np.int64)
    assert spars(sizes_host=wrong_sizes.ctypes.data) == B.DEFT_EINVAL
    assert spars(sumsq_pinned=0) == B.DEFT_EINVAL
    assert spars(idx_out_dev=0) == B.DEFT_EINVAL
    assert spars(ws_dev=0x4004) == B.DEFT_EINVAL
    assert spars(ws_bytes=64) == B.DEFT_EWS
    assert cnt.value == -7 and kr.value == -7
    ok_job = B.DeftJob(N=16, L=2, n_workers=2, rank=0, launch_shape=0, d=0.25,
                       offsets_host=off.ctypes.data, offsets_dev=0x5000,
                       sizes_host=sizes.ctypes.data, sumsq_pinned=0x6000,
                       norms_host=bufs["norms"].ctypes.data, k_host=bufs["k"].ctypes.data,
                       owner_bin_host=bufs["owner"].ctypes.data,
                       my_layers_host=bufs["mine"].ctypes.data, seg_off_host=bufs["seg"].ctypes.data,
                       idx_out_dev=0x2000, val_out_dev=0x3000, out_cap=16, ws_dev=0x4000,
                       ws_bytes=1 << 20)

    def accsp(e=0x1000, gr=0x7000, acc=0x8000):
        return lib.deft_accumulate_sparsify(C.addressof(ok_job), C.c_void_p(e), C.c_void_p(gr), 0.5,
                                            C.c_void_p(acc), 0, None, None, C.addressof(cnt),
                                            C.addressof(kr))

    assert accsp(gr=0) == B.DEFT_EINVAL
    assert accsp(acc=0) == B.DEFT_EINVAL
    assert accsp(e=0) == B.DEFT_EINVAL
    assert accsp(gr=0x7004) == B.DEFT_EINVAL
    assert accsp(acc=0x8008) == B.DEFT_EINVAL

    def topk(g=0x1000, N=16, K=4, idx=0x2000, val=0x3000, ws=0x4000, wsb=1 << 20, shape=0):
        return lib.topk_global(C.c_void_p(g), N, K, C.c_void_p(idx), C.c_void_p(val),
                               C.c_void_p(ws), wsb, shape, None)

    assert topk(shape=5) == B.DEFT_EINVAL
    assert topk(K=17) == B.DEFT_EINVAL
    assert topk(K=-1) == B.DEFT_EINVAL
    assert topk(N=2 ** 31) == B.DEFT_ERANGE
    assert topk(wsb=0) == B.DEFT_EWS
    assert topk(K=0) == B.DEFT_OK
    assert topk(idx=0) == B.DEFT_EINVAL


def test_total_k_and_cltk_leader_hand_values(deft):
    """Alg. 3's first statement and the turn-taking rule of cyclic local Top-k (Sec. 3.1), by
    hand: 11689512 * 0.01 = 116895.12 -> 116895; 150 * 0.01 = 1.5 -> 2 (half up)."""
    B = deft
    assert B.deft_total_k(11689512, 0.01) == 116895
    assert B.deft_total_k(150, 0.01) == 2
    assert B.deft_total_k(10, 1.0) == 10
    for N, d in [(300938, 0.01), (19780400, 0.001), (7, 0.5), (354823168, 0.001)]:
        assert B.deft_total_k(N, d) == O.total_k(N, d)
    with pytest.raises(B.DeftError):
        B.deft_total_k(0, 0.5)
    with pytest.raises(B.DeftError):
        B.deft_total_k(10, 1.5)
    assert [B.deft_cltk_leader(t, 4) for t in range(6)] == [0, 1, 2, 3, 0, 1]
    assert B.deft_cltk_leader(9, 1) == 0
    with pytest.raises(B.DeftError):
        B.deft_cltk_leader(-1, 4)


def test_partition_hand_worked_five_tensors(deft):
    """The library against the same pencil-worked case of Alg. 2 that pins the oracle
    (tests/test_oracle_pins.py): tensors 23, 5, 12, 1, 9."""
    B = deft
    off, lt = B.deft_partition([23, 5, 12, 1, 9], 4)
    assert off.tolist() == [0, 6, 12, 18, 23, 28, 40, 41, 50] and lt.tolist() == [0, 0, 0, 0, 1, 2, 3, 4]
    off, lt = B.deft_partition([23, 5, 12, 1, 9], 5)
    assert off.tolist() == [0, 5, 10, 15, 19, 23, 28, 31, 34, 36, 38, 40, 41, 50]
    assert lt.tolist() == [0, 0, 0, 0, 0, 1, 2, 2, 2, 2, 2, 3, 4]
    off, _ = B.deft_partition([0, 2, 0], 4)   # 2 > 2/4 is cut in four; the empty pieces vanish
    assert off.tolist() == [0, 1, 2]


def test_cost_model_hand_worked(deft):
    """deft_cost_model against the pencil values of Eq. 3-8 (see the oracle's pin of the same
    two cases for the working)."""
    B = deft
    a = B.deft_cost_model([100, 50, 200, 10], [4, 2, 8, 1], [1, 1, 0, 1], 2, 360, 15)
    assert a["C_i"] == pytest.approx([415.8883, 173.2868], abs=1e-4)
    assert a["f_n"] == pytest.approx(2.34413, abs=1e-5)
    assert a["f_trivial"] == pytest.approx(2.68802, abs=1e-5)
    b = B.deft_cost_model([64, 32, 16, 8, 8], [16, 8, 4, 2, 2], [0, 1, 2, 1, 2], 3, 128, 32)
    assert b["f_n"] == pytest.approx(2.5, rel=1e-12)
    assert b["C_trivial"] == pytest.approx(100.9973, abs=1e-4)


def test_host_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """csrc/deft_host.cpp built with the host compiler under -fsanitize=address,undefined and
    driven by tests/host_sanitize_check.c over 400 seeded shapes with exactly-sized output
    arrays: any out-of-bounds access or undefined operation aborts the run with a report."""
    import shutil
    import subprocess
    cxx, cc = shutil.which("g++"), shutil.which("gcc")
    if not cxx or not cc:
        pytest.skip("no host compiler")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include")]
    obj_lib, obj_drv, exe = (str(tmp_path / n) for n in ("deft_host.o", "driver.o", "host_sanitize"))
    subprocess.run([cxx, "-std=c++17", "-ffp-contract=off", *san, *inc, "-c",
                    os.path.join(ROOT, "paper_2307_03500_amd", "csrc", "deft_host.cpp"),
                    "-o", obj_lib], check=True)
    subprocess.run([cc, "-std=c99", *san, *inc, "-c",
                    os.path.join(ROOT, "tests", "host_sanitize_check.c"), "-o", obj_drv], check=True)
    # the run-time is linked statically so that it is first in the library list whatever the
    # environment preloads
    subprocess.run([cxx, "-fsanitize=address,undefined", "-static-libasan", obj_lib, obj_drv,
                    "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stderr[-2000:]
    assert "host sanitize ok" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
