"""The library's HIP kernels and host code compiled for the CPU (tests/cpu_emulation) and

  * compared with the oracle through the same C ABI (forward, backward, update, fused update, plan
    arrays, both arms) -- the kernels' logic is checked here without a GPU;
  * run under AddressSanitizer + UBSan, single-table and batched, on seeded inputs: any
    out-of-bounds or misaligned access of a kernel fails the test.  The batched entry points, which
    are switched off in the GPU build, are switched on in this build.

Nothing here stands in for the GPU parity tests: the emulation runs one workgroup at a time and
knows nothing about the hardware's memory system."""
import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest

import tt_workloads as wl

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "cpu_emulation"))
import build as emu_build  # noqa: E402

BUILD_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cpu_emulation", "_build")
pytestmark = pytest.mark.skipif(not emu_build.available(), reason="host clang++ of the ROCm toolchain not found")


@pytest.fixture(scope="module")
def emu():
    from paper_2507_14668_amd import binding
    lib = ctypes.CDLL(emu_build.build_shared(BUILD_DIR))
    vp, i64, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float
    lib.tt_workspace_bytes.restype = ctypes.c_size_t
    lib.tt_workspace_bytes.argtypes = [vp, i64, i64]
    lib.tt_index_reorder.argtypes = [vp, vp, vp, i64, i64, vp, vp, ctypes.c_size_t, vp, vp]
    lib.tt_emb_bag_forward.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp]
    lib.tt_emb_bag_backward.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp]
    lib.tt_core_sgd_update.argtypes = [vp, vp, vp, f32, vp]
    lib.tt_emb_bag_backward_sgd.argtypes = [vp, vp, vp, vp, i64, i64, vp, f32, vp]
    return lib, binding


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _aligned(nbytes):
    raw = np.empty(nbytes + 256, dtype=np.uint8)
    off = (-raw.ctypes.data) % 256
    return raw[off:off + nbytes]


def _table(binding, shape, cores):
    t = binding.CTable()
    t.num_rows = shape.num_rows
    t.n[:], t.d[:], t.r[:] = shape.n, shape.d, shape.r
    for k in range(3):
        t.core[k] = cores[k].ctypes.data
    return t


def _run(emu, shape, cores, idx, off, grad, lr):
    lib, binding = emu
    cores = [np.ascontiguousarray(c, dtype=np.float32).copy() for c in cores]
    idx, off = np.ascontiguousarray(idx, dtype=np.int64), np.ascontiguousarray(off, dtype=np.int64)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    nnz, nb = len(idx), len(off) - 1
    table = _table(binding, shape, cores)
    ws = _aligned(lib.tt_workspace_bytes(ctypes.byref(table), nnz, nb))
    plan = binding.CPlan()
    assert lib.tt_index_reorder(ctypes.byref(table), _ptr(idx), _ptr(off), nnz, nb, None, _ptr(ws), ws.nbytes,
                                ctypes.byref(plan), None) == 0
    res = {}

    def ints(name, count):
        o = getattr(plan, name) - ws.ctypes.data
        return ws[o:o + 4 * count].view(np.int32).copy()

    counts = ints("counts", 16)
    ur, up = int(counts[0]), int(counts[1])
    res["plan_arrays"] = dict(U_r=ur, U_p=up, num_valid=int(counts[2]), status=int(counts[4]), uniq_row=ints("uniq_row", ur),
                       row_seg=ints("row_seg", ur + 1), uniq_pref=ints("uniq_pref", up), pref_seg=ints("pref_seg", up + 1),
                       lookup2row=ints("lookup2row", nnz), i2_seg=ints("i2_seg", shape.n[1] + 1),
                       i3_seg=ints("i3_seg", shape.n[2] + 1), i1_seg=ints("i1_seg", shape.n[0] + 1))
    for arm, pl in (("plan", ctypes.byref(plan)), ("naive", None)):
        out = np.full((nb, shape.dim), np.nan, dtype=np.float32)
        assert lib.tt_emb_bag_forward(ctypes.byref(table), pl, _ptr(idx), _ptr(off), nnz, nb, _ptr(out), None) == 0
        dg = [np.full_like(c, np.nan) for c in cores]
        arr = (ctypes.c_void_p * 3)(*[g.ctypes.data for g in dg])
        assert lib.tt_emb_bag_backward(ctypes.byref(table), pl, _ptr(idx), _ptr(off), nnz, nb, _ptr(grad), arr, None) == 0
        res[arm] = (out, dg)
    # update (touched slices) after the planned backward, and the fused call on fresh cores
    dg = res["plan"][1]
    arr = (ctypes.c_void_p * 3)(*[g.ctypes.data for g in dg])
    upd = [c.copy() for c in cores]
    t_upd = _table(binding, shape, upd)
    assert lib.tt_core_sgd_update(ctypes.byref(t_upd), ctypes.byref(plan), arr, ctypes.c_float(lr), None) == 0
    fused = [c.copy() for c in cores]
    t_fused = _table(binding, shape, fused)
    assert lib.tt_emb_bag_backward_sgd(ctypes.byref(t_fused), ctypes.byref(plan), _ptr(idx), _ptr(off), nnz, nb,
                                       _ptr(grad), ctypes.c_float(lr), None) == 0
    res["updated"], res["fused"] = upd, fused
    return res


@pytest.mark.parametrize("name,n,d,r,nb,ml", [
    ("plain", (5, 4, 6), (2, 3, 2), (1, 3, 5, 1), 150, 6),
    ("mfma_r32_split", (9, 3, 5), (4, 8, 4), (1, 32, 32, 1), 260, 5),   # 3 core-1 slices: split workgroups
    ("mfma_r64_two_strips", (3, 2, 11), (4, 8, 4), (1, 64, 64, 1), 120, 4),
    # rows looked up hundreds of times: segments of the gradient merge that span whole workgroups of stage 1
    ("mfma_r64_hot_rows", (2, 1, 2), (4, 8, 4), (1, 64, 64, 1), 800, 4),
    ("plain_hot_rows", (1, 2, 2), (2, 3, 2), (1, 3, 5, 1), 2500, 3),
    # more than 64 prefixes under one i2 (the staged plan entries are refilled) and prefixes with more
    # than 32 distinct rows (row batches that cut a prefix's rows at any position)
    ("mfma_r32_refill", (75, 1, 3), (4, 8, 4), (1, 32, 32, 1), 400, 3),
    ("mfma_r64_row_batches", (2, 2, 45), (4, 8, 4), (1, 64, 64, 1), 300, 4),
    # row factors above 1023: the groupings by i2 / i3 become radix sorts of more than one digit
    ("mfma_r32_wide_n2", (1, 2100, 2), (4, 8, 4), (1, 32, 32, 1), 200, 3),
    ("plain_wide_n3", (2, 1, 1500), (2, 3, 2), (1, 3, 5, 1), 300, 3),
    # 31-bit row keys (2.1e9 rows): four radix passes
    ("plain_31_bit_keys", (1290, 1290, 1290), (2, 3, 2), (1, 3, 5, 1), 300, 4),
])
def test_emulated_kernels_match_oracle(emu, ora, name, n, d, r, nb, ml):
    import gpu_util as g
    shape, cores, idx, off, grad = wl.small_random_problem(301, n=n, d=d, r=r, num_bags=nb, max_len=ml, sigma=0.2)
    lr = 0.05
    res = _run(emu, shape, cores, idx, off, grad, lr)
    ref_plan = ora.reorder_plan(shape, idx, off)
    p = res["plan_arrays"]
    assert p["status"] == 0 and p["num_valid"] == ref_plan["num_valid"]
    for key in ("uniq_row", "row_seg", "uniq_pref", "pref_seg", "lookup2row"):
        assert np.array_equal(p[key], ref_plan[key]), key
    i3 = np.sort(ref_plan["uniq_row"] % shape.n[2])
    assert np.array_equal(p["i3_seg"], np.searchsorted(i3, np.arange(shape.n[2] + 1)))
    i2 = np.sort(ref_plan["uniq_pref"] % shape.n[1])
    assert np.array_equal(p["i2_seg"], np.searchsorted(i2, np.arange(shape.n[1] + 1)))
    assert np.array_equal(p["i1_seg"], np.searchsorted(ref_plan["uniq_pref"] // shape.n[1], np.arange(shape.n[0] + 1)))
    ref_out = ora.forward(shape, cores, idx, off)
    ref_dg = ora.backward(shape, cores, idx, off, grad)
    for arm in ("plan", "naive"):
        out, dg = res[arm]
        g.assert_close_rows(out, ref_out, g.FWD_RTOL, shape.dim, "%s forward (%s)" % (name, arm))
        g.assert_grads_close(shape, dg, ref_dg, what="%s dG (%s)" % (name, arm))
    g.assert_grads_close(shape, res["updated"], ora.sgd(cores, ref_dg, lr), what="%s updated G" % name)
    for k in range(3):
        assert np.array_equal(res["fused"][k], res["updated"][k]), "fused update differs from backward + update"


def test_emulated_one_hot_batch_and_mixed_bag_lengths(emu, ora):
    """One lookup per bag (the bag sum takes four bags of a lane group at a time) and a batch whose bags
    hold zero or one lookup (the fast path gives way to the general one wherever a bag is not single)."""
    import gpu_util as g
    shape, cores, _, _, _ = wl.small_random_problem(41, n=(5, 4, 6), d=(2, 3, 2), r=(1, 3, 5, 1))
    rng = np.random.default_rng(5)
    sparse = np.zeros(4000, np.int64)  # runs of more than a tile's worth of empty bags between the lookups
    sparse[[0, 1500, 1501, 3999]] = (3, 2, 1200, 4)
    for nb, lens in ((1500, None), (1100, rng.integers(0, 2, 1100)), (4000, sparse)):
        lens = np.ones(nb, np.int64) if lens is None else lens
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        idx = rng.integers(0, shape.num_rows, int(off[-1])).astype(np.int64)
        grad = rng.standard_normal(nb * shape.dim).astype(np.float32)
        res = _run(emu, shape, cores, idx, off, grad, 0.05)
        ref_out = ora.forward(shape, cores, idx, off)
        assert np.array_equal(res["plan_arrays"]["lookup2row"], ora.reorder_plan(shape, idx, off)["lookup2row"])
        for arm in ("plan", "naive"):
            g.assert_close_rows(res[arm][0], ref_out, g.FWD_RTOL, shape.dim, "one-hot forward (%s)" % arm)
        g.assert_grads_close(shape, res["plan"][1], ora.backward(shape, cores, idx, off, grad), what="one-hot dG")


@pytest.mark.parametrize("nb,ml,rows,hot,max_group", [(300, 9, 400, 5, 64), (40, 300, 3000, 0, 16), (200, 5, 50, 45, 64)])
def test_emulated_index_graph_edges_match_oracle(emu, ora, nb, ml, rows, hot, max_group):
    """The edge-generation job (pairs per bag, two stable radix sorts, run heads) against the loop oracle:
    short bags, bags longer than a wavefront round and than the per-bag cap, almost every row hot."""
    lib, _ = emu
    rng = np.random.default_rng(nb)
    lens = rng.integers(0, ml + 1, nb)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.minimum((rows ** rng.random(int(off[-1]))).astype(np.int64), rows - 1)  # skewed
    idx[::17] = -1
    rank = rng.permutation(rows).astype(np.int32)
    ref = ora.index_graph_edges(idx, off, rank, hot, max_group)
    cap = max(1, int(sum(min(l, max_group) * (min(l, max_group) - 1) // 2 for l in lens)))
    lib.tt_index_graph_workspace_bytes.restype = ctypes.c_size_t
    lib.tt_index_graph_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    ws = _aligned(lib.tt_index_graph_workspace_bytes(nb, cap))
    eu, ev, ew = (np.full(cap, -1, np.int32) for _ in range(3))
    counts = np.zeros(4, np.int32)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    lib.tt_index_graph_edges.argtypes = [vp, vp, i64, i64, vp, i64, i64, ctypes.c_int32, vp, ctypes.c_size_t, i64,
                                         vp, vp, vp, vp, vp]
    assert lib.tt_index_graph_edges(_ptr(idx), _ptr(off), len(idx), nb, _ptr(rank), rows, hot, max_group, _ptr(ws),
                                    ws.nbytes, cap, _ptr(eu), _ptr(ev), _ptr(ew), _ptr(counts), None) == 0
    assert counts[2] == 0 and counts[0] == sum(ref.values()) and counts[1] == len(ref)
    got = {(int(u), int(v)): int(w) for u, v, w in zip(eu[:counts[1]], ev[:counts[1]], ew[:counts[1]])}
    assert got == ref
    keys = list(zip(eu[:counts[1]].tolist(), ev[:counts[1]].tolist()))
    assert keys == sorted(keys), "edges must come out sorted by (u, v)"
    # a capacity that is too small is reported, and nothing is produced
    if sum(ref.values()) > 1:
        assert lib.tt_index_graph_edges(_ptr(idx), _ptr(off), len(idx), nb, _ptr(rank), rows, hot, max_group, _ptr(ws),
                                        ws.nbytes, sum(ref.values()) - 1, _ptr(eu), _ptr(ev), _ptr(ew), _ptr(counts), None) == 0
        assert counts[2] == 1 and counts[1] == 0


@pytest.fixture(scope="module")
def asan_harness():
    return emu_build.build_harness(BUILD_DIR, "address")


@pytest.mark.parametrize("kind,shuffle", [("mfma", None), ("plain", None), ("unaligned", None), ("wide", None), ("keys31", None),
                                          ("mfma", "11"), ("plain", "12")])
def test_sanitized_single_and_batched_calls(asan_harness, kind, shuffle):
    """Every entry point under AddressSanitizer + UBSan.  While a launch runs, the host structs of the
    C ABI (tables, plans, batch items) and the library's host copies of the table descriptors are
    poisoned: a kernel that followed a host pointer -- harmless on the CPU, a fault on a GPU -- is
    reported.  With `shuffle` the workgroups of every launch run in a seeded random order over both grid
    dimensions, so that the tables of a batched launch are interleaved."""
    env = dict(os.environ, ASAN_OPTIONS="detect_stack_use_after_return=0:detect_leaks=0", UBSAN_OPTIONS="halt_on_error=1")
    if shuffle:
        env["EMU_SHUFFLE"] = shuffle
    # the kinds with very wide tables run the planned arm only: a dense update sweep over their cores
    # takes the emulation minutes and is no other code than on the small tables
    planned_only = kind in ("wide", "keys31")
    res = subprocess.run([asan_harness, kind] + (["1"] if planned_only else []), capture_output=True, text=True, env=env,
                         timeout=600)
    text = res.stdout + res.stderr
    assert res.returncode == 0, text[-4000:]
    assert "ERROR" not in text and "runtime error" not in text, text[-4000:]
    assert text.count("identical") == (1 if planned_only else 2), text[-2000:]  # per arm: batched == single-table
    assert ", 0 values off" in text, text[-2000:]  # the same tables as one fused table: same results to rounding


def test_emulated_kernels_on_random_shapes(emu, ora):
    """Seeded random shapes within the library's limits (ranks and factors that are not powers of
    two, single-slice cores, padded row counts, the matrix-core shapes): every arm against the
    oracle, and the fused update bit for bit against backward + update."""
    import gpu_util as g
    rng = np.random.default_rng(20250714)
    for case in range(14):
        while True:
            n = tuple(int(x) for x in rng.integers(1, 9, size=3))
            d = tuple(int(x) for x in rng.choice([1, 2, 3, 4, 5, 8], size=3))
            r1, r2 = int(rng.choice([1, 2, 3, 7, 16, 33, 64])), int(rng.choice([1, 2, 5, 8, 17, 32, 64]))
            if rng.random() < 0.25:
                d, r1 = (4, 8, 4), int(rng.choice([32, 64]))
                r2 = r1
            dim, p12, s2 = d[0] * d[1] * d[2], d[0] * d[1] * r2, d[1] * r2
            lds = d[0] * r1 + d[0] * d[1] * (r2 | 1) + p12 + dim + 8 * r2 * d[2]
            if dim <= 1024 and p12 <= 4096 and s2 <= 4096 and lds * 4 <= 65536:
                break
        cap = n[0] * n[1] * n[2]
        num_rows = int(rng.integers(max(1, cap - n[2] + 1), cap + 1))
        nb, ml = int(rng.integers(1, 100)), int(rng.integers(1, 8))
        shape, cores, idx, off, grad = wl.small_random_problem(7000 + case, n=n, d=d, r=(1, r1, r2, 1), num_rows=num_rows,
                                                              num_bags=nb, max_len=ml, sigma=0.3)
        what = "n=%s d=%s r=(%d,%d) rows=%d" % (n, d, r1, r2, num_rows)
        res = _run(emu, shape, cores, idx, off, grad, 0.05)
        ref_out, ref_dg = ora.forward(shape, cores, idx, off), ora.backward(shape, cores, idx, off, grad)
        for arm in ("plan", "naive"):
            out, dg = res[arm]
            g.assert_close_rows(out, ref_out, g.FWD_RTOL, shape.dim, "%s forward (%s)" % (what, arm))
            g.assert_grads_close(shape, dg, ref_dg, what="%s dG (%s)" % (what, arm))
        for k in range(3):
            assert np.array_equal(res["fused"][k], res["updated"][k]), what


def test_results_do_not_depend_on_workgroup_order(asan_harness):
    """The emulation runs the workgroups of a launch one after the other; last to first must give
    the same bits as first to last (no kernel relies on another workgroup of its launch)."""
    sums = []
    for reverse in (False, True):
        env = dict(os.environ, ASAN_OPTIONS="detect_stack_use_after_return=0:detect_leaks=0", UBSAN_OPTIONS="halt_on_error=1")
        if reverse:
            env["EMU_REVERSE"] = "1"
        res = subprocess.run([asan_harness, "mfma"], capture_output=True, text=True, env=env, timeout=900)
        text = res.stdout + res.stderr
        assert res.returncode == 0 and "ERROR" not in text, text[-3000:]
        sums.append([ln for ln in text.splitlines() if ln.startswith("checksum")])
    # first checksum: the planned arm (no atomics, must not move); second: the naive arm, whose
    # backward adds with float atomics in arrival order and is not expected to be bit-stable
    assert len(sums[0]) == 2 and sums[0][0] == sums[1][0]
