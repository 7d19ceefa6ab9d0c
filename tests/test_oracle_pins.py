"""Pins of the CPU oracle against things other than itself (CPU only).

Each test ties one part of `oracle/` to a value the paper prints, a closed
form, a library routine the special case reduces to, or an exact identity, so
that a dropped term, a wrong index order or a transposed operand fails here.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import tt_workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def cores_nd(shape, cores):
    g1 = np.asarray(cores[0], dtype=np.float64).reshape(shape.n[0], shape.d[0], shape.r[1])
    g2 = np.asarray(cores[1], dtype=np.float64).reshape(shape.r[1], shape.n[1], shape.d[1], shape.r[2])
    g3 = np.asarray(cores[2], dtype=np.float64).reshape(shape.r[2], shape.n[2], shape.d[2])
    return g1, g2, g3


def dense_table(shape, cores):
    """W[N_pad, D] straight from the TT-matrix definition with a library einsum."""
    g1, g2, g3 = cores_nd(shape, cores)
    w = np.einsum("ipb,bjqc,ckr->ijkpqr", g1, g2, g3)
    return w.reshape(shape.n[0] * shape.n[1] * shape.n[2], shape.dim)


# ---------------------------------------------------------------- index split
def test_index_example_printed_in_paper(ora):
    rows = [l for l in open(os.path.join(GOLDEN, "index_example.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 2
    for line in rows:
        n, row, tt = [p.split() for p in line.split("|")]
        assert ora.split_index(int(row[0]), [int(x) for x in n]) == tuple(int(x) for x in tt)


def test_index_split_round_trip_and_digit_order(ora):
    n = (3, 4, 5)
    seen = set()
    for i in range(60):
        i1, i2, i3 = ora.split_index(i, n)
        assert 0 <= i1 < 3 and 0 <= i2 < 4 and 0 <= i3 < 5
        assert (i1 * n[1] + i2) * n[2] + i3 == i  # i1 is the most significant digit
        seen.add((i1, i2, i3))
    assert len(seen) == 60
    # brute force: the lexicographic enumeration of digits is the row order
    for i, t in enumerate(itertools.product(range(3), range(4), range(5))):
        assert ora.split_index(i, n) == t


# ----------------------------------------------------------------------- rows
@pytest.mark.parametrize("seed,n,d,r", [(1, (3, 4, 5), (2, 3, 2), (1, 3, 4, 1)),
                                        (2, (2, 2, 2), (2, 2, 2), (1, 2, 2, 1)),
                                        (3, (5, 2, 3), (1, 4, 3), (1, 5, 2, 1))])
def test_rows_equal_dense_materialisation(ora, seed, n, d, r):
    shape, cores, *_ = wl.small_random_problem(seed, n=n, d=d, r=r)
    w = dense_table(shape, cores)
    for i in range(shape.num_rows):
        np.testing.assert_allclose(ora.row(shape, cores, i), w[i], rtol=1e-12, atol=1e-14)


def test_rows_config1_shape_equal_dense_materialisation(ora):
    cfg = wl.get_config(1)
    shape, cores = cfg.tables[0], wl.make_cores(cfg, 0)
    w = dense_table(shape, cores)
    assert w.shape == (1000, 16)
    idx = np.arange(1000, dtype=np.int64)
    out = ora.forward(shape, cores, idx, np.arange(1001, dtype=np.int64))
    np.testing.assert_allclose(out, w, rtol=1e-6, atol=1e-9)


def test_rank_one_is_kronecker_product(ora):
    shape, cores, *_ = wl.small_random_problem(7, n=(3, 2, 4), d=(2, 3, 4), r=(1, 1, 1, 1))
    g1, g2, g3 = cores_nd(shape, cores)
    for i in range(shape.num_rows):
        i1, i2, i3 = ora.split_index(i, shape.n)
        closed = np.kron(np.kron(g1[i1, :, 0], g2[0, i2, :, 0]), g3[0, i3, :])
        np.testing.assert_allclose(ora.row(shape, cores, i), closed, rtol=1e-14)


# -------------------------------------------------------------------- forward
def test_forward_equals_library_embedding_bag_on_dense_table(ora):
    shape, cores, idx, off, _ = wl.small_random_problem(11, num_bags=40, max_len=6)
    assert (np.diff(off) == 0).any(), "fixture must contain an empty bag"
    w = torch.from_numpy(dense_table(shape, cores))
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(idx), w, torch.from_numpy(off[:-1]),
                                            mode="sum")
    for dedup in (False, True):
        out = ora.forward(shape, cores, idx, off, dedup=dedup)
        np.testing.assert_allclose(out, ref.numpy(), rtol=2e-6, atol=1e-7)
        assert np.all(out[np.diff(off) == 0] == 0.0)


def test_forward_duplicates_count_twice(ora):
    shape, cores, *_ = wl.small_random_problem(12)
    w = dense_table(shape, cores)
    out = ora.forward(shape, cores, [5, 5, 9], [0, 3])
    np.testing.assert_allclose(out[0], 2 * w[5] + w[9], rtol=2e-6, atol=1e-7)


def test_forward_invariances(ora):
    shape, cores, idx, off, _ = wl.small_random_problem(13, num_bags=25, max_len=7)
    out = ora.forward(shape, cores, idx, off)
    rng = np.random.default_rng(0)
    # (i) order of the lookups inside a bag does not matter (up to rounding)
    idx2 = idx.copy()
    for b in range(len(off) - 1):
        seg = idx2[off[b]:off[b + 1]]
        rng.shuffle(seg)
    np.testing.assert_allclose(ora.forward(shape, cores, idx2, off), out, rtol=1e-6, atol=1e-7)
    # (ii) permuting bags permutes the output rows, bit for bit
    perm = rng.permutation(len(off) - 1)
    lens = np.diff(off)
    off_p = np.concatenate([[0], np.cumsum(lens[perm])])
    idx_p = np.concatenate([idx[off[b]:off[b + 1]] for b in perm] + [np.zeros(0, np.int64)])
    out_p = ora.forward(shape, cores, idx_p, off_p)
    assert np.array_equal(out_p, out[perm])
    # (iii) definition mode and dedup mode agree
    np.testing.assert_allclose(ora.forward(shape, cores, idx, off, dedup=True), out, rtol=1e-6, atol=1e-7)


def test_prefix_reuse_identity_on_the_papers_two_index_bag(ora):
    """Bag {0,1} of the 2x2x2 example: both rows share (i1,i2) = (0,0), so the bag sum is
    Slice1 x Slice2 x (Slice3[0] + Slice3[1]) -- the reuse equation of Section III-B."""
    shape, cores, *_ = wl.small_random_problem(21, n=(2, 2, 2), d=(2, 3, 2), r=(1, 3, 2, 1))
    g1, g2, g3 = cores_nd(shape, cores)
    p12 = np.einsum("pb,bqc->pqc", g1[0], g2[:, 0])
    reuse = np.einsum("pqc,cr->pqr", p12, g3[:, 0] + g3[:, 1]).reshape(-1)
    out = ora.forward(shape, cores, [1, 0], [0, 2])
    np.testing.assert_allclose(out[0], reuse, rtol=2e-6, atol=1e-7)


def test_sample_reuse_route_equals_dense_table_and_counts_groups(ora):
    """The sample-level evaluation order (one chain per (bag, prefix), core-3 slices summed first)
    against the library embedding_bag on the dense table, and its group count against a brute-force
    count of distinct (bag, row div n3) pairs.  Bags here hold several rows of one prefix, repeated
    rows, an empty bag and an invalid index."""
    shape, cores, idx, off, _ = wl.small_random_problem(14, n=(2, 3, 6), num_bags=30, max_len=9)
    idx = idx.copy()
    idx[3] = -1
    assert (np.diff(off) == 0).any()
    w = dense_table(shape, cores)
    ref = np.zeros((len(off) - 1, shape.dim))
    pairs = set()
    for b in range(len(off) - 1):
        for i in idx[off[b]:off[b + 1]]:
            if 0 <= i < shape.num_rows:
                ref[b] += w[i]
                pairs.add((b, int(i) // shape.n[2]))
    out, groups = ora.forward_sample_reuse(shape, cores, idx, off)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    assert groups == len(pairs) < int(((idx >= 0) & (idx < shape.num_rows)).sum()), "fixture must share prefixes inside bags"


# ------------------------------------------------------------------- backward
def dense_route_grads(shape, cores, idx, off, grad):
    """dL/dW by scatter-add, then contracted with the other two cores (library einsum)."""
    g1, g2, g3 = cores_nd(shape, cores)
    n1, n2, n3 = shape.n
    d1, d2, d3 = shape.d
    dw = np.zeros((n1 * n2 * n3, shape.dim))
    g = np.asarray(grad, dtype=np.float64).reshape(-1, shape.dim)
    for b in range(len(off) - 1):
        for l in range(off[b], off[b + 1]):
            dw[idx[l]] += g[b]
    dw = dw.reshape(n1, n2, n3, d1, d2, d3)
    dg1 = np.einsum("ijkpqr,bjqc,ckr->ipb", dw, g2, g3)
    dg2 = np.einsum("ijkpqr,ipb,ckr->bjqc", dw, g1, g3)
    dg3 = np.einsum("ijkpqr,ipb,bjqc->ckr", dw, g1, g2)
    return [dg1.reshape(-1), dg2.reshape(-1), dg3.reshape(-1)]


@pytest.mark.parametrize("dedup", [False, True])
def test_backward_equals_dense_route(ora, dedup):
    shape, cores, idx, off, grad = wl.small_random_problem(31, num_bags=30, max_len=6)
    ref = dense_route_grads(shape, cores, idx, off, grad)
    got = ora.backward(shape, cores, idx, off, grad, dedup=dedup)
    for k in range(3):
        np.testing.assert_allclose(got[k], ref[k], rtol=1e-5, atol=1e-6)


def test_backward_equals_torch_autograd(ora):
    shape, cores, idx, off, grad = wl.small_random_problem(32, n=(4, 3, 2), d=(3, 2, 2), r=(1, 2, 5, 1),
                                                          num_bags=20)
    t = [torch.tensor(np.asarray(c, dtype=np.float64), requires_grad=True) for c in cores]
    g1 = t[0].reshape(shape.n[0], shape.d[0], shape.r[1])
    g2 = t[1].reshape(shape.r[1], shape.n[1], shape.d[1], shape.r[2])
    g3 = t[2].reshape(shape.r[2], shape.n[2], shape.d[2])
    w = torch.einsum("ipb,bjqc,ckr->ijkpqr", g1, g2, g3).reshape(-1, shape.dim)
    out = torch.nn.functional.embedding_bag(torch.from_numpy(idx), w, torch.from_numpy(off[:-1]), mode="sum")
    out.backward(torch.from_numpy(grad.astype(np.float64)).reshape(-1, shape.dim))
    got = ora.backward(shape, cores, idx, off, grad)
    for k in range(3):
        np.testing.assert_allclose(got[k], t[k].grad.numpy(), rtol=1e-5, atol=1e-6)


def loss(ora, shape, cores, idx, off, grad):
    out = ora.forward(shape, cores, idx, off).astype(np.float64)
    return float((out * np.asarray(grad, dtype=np.float64).reshape(out.shape)).sum())


def test_backward_finite_difference_is_exact_by_multilinearity(ora):
    """L = sum_b <out_b, g_b> is linear in each core, so a one-sided difference with any step
    is exact (up to the fp32 rounding of the oracle's stored outputs)."""
    shape, cores, idx, off, grad = wl.small_random_problem(33, num_bags=15)
    dg = ora.backward(shape, cores, idx, off, grad)
    base = loss(ora, shape, cores, idx, off, grad)
    rng = np.random.default_rng(5)
    for k in range(3):
        for e in rng.choice(cores[k].size, size=6, replace=False):
            pert = [c.copy() for c in cores]
            pert[k][e] += np.float32(0.5)
            fd = (loss(ora, shape, pert, idx, off, grad) - base) / 0.5
            assert abs(fd - dg[k][e]) <= 2e-4 * max(1.0, abs(dg[k][e])), (k, e, fd, dg[k][e])


def test_backward_euler_identity(ora):
    """Each row is homogeneous of degree 1 in every core, hence <dG_k, G_k> = L for k = 1,2,3."""
    shape, cores, idx, off, grad = wl.small_random_problem(34, num_bags=50, max_len=8)
    dg = ora.backward(shape, cores, idx, off, grad)
    base = loss(ora, shape, cores, idx, off, grad)
    for k in range(3):
        inner = float(np.dot(dg[k].astype(np.float64), np.asarray(cores[k], dtype=np.float64)))
        assert abs(inner - base) <= 1e-5 * max(1.0, abs(base))


def test_backward_repeated_rows_sum(ora):
    """Listing a bag c times equals scaling its gradient by c (gradients of repeats add up)."""
    shape, cores, *_ = wl.small_random_problem(35)
    g = np.random.default_rng(1).standard_normal(shape.dim).astype(np.float32)
    three = ora.backward(shape, cores, [7, 7, 7], [0, 1, 2, 3], np.tile(g, 3))
    once = ora.backward(shape, cores, [7], [0, 1], 3.0 * g)
    for k in range(3):
        np.testing.assert_allclose(three[k], once[k], rtol=1e-6, atol=1e-7)


def test_untouched_slices_have_zero_gradient(ora):
    shape, cores, *_ = wl.small_random_problem(36)
    g = np.ones(shape.dim, dtype=np.float32)
    dg = ora.backward(shape, cores, [0], [0, 1], g)
    d1 = dg[0].reshape(shape.n[0], -1)
    assert np.all(d1[1:] == 0.0) and np.any(d1[0] != 0.0)
    d3 = dg[2].reshape(shape.r[2], shape.n[2], shape.d[2])
    assert np.all(d3[:, 1:, :] == 0.0)


# ------------------------------------------------------------------------ SGD
def test_sgd_closed_form_and_descent(ora):
    shape, cores, idx, off, grad = wl.small_random_problem(41, num_bags=20)
    dg = ora.backward(shape, cores, idx, off, grad)
    same = ora.sgd(cores, dg, 0.0)
    for k in range(3):
        assert np.array_equal(same[k], cores[k])
    lr = 1e-3
    new = ora.sgd(cores, dg, lr)
    for k in range(3):
        expect = (cores[k].astype(np.float64) - np.float64(np.float32(lr)) * dg[k].astype(np.float64))
        assert np.array_equal(new[k], expect.astype(np.float32))
    l0 = loss(ora, shape, cores, idx, off, grad)
    l1 = loss(ora, shape, new, idx, off, grad)
    first_order = lr * sum(float(np.dot(d.astype(np.float64), d.astype(np.float64))) for d in dg)
    assert l1 < l0
    assert abs((l0 - l1) - first_order) <= 0.05 * first_order


# ----------------------------------------------------------------------- plan
def test_reorder_plan_matches_brute_force(ora):
    shape, cores, idx, off, _ = wl.small_random_problem(51, num_bags=30, max_len=6)
    idx = idx.copy()
    idx[3] = -1
    idx[10] = shape.num_rows  # two invalid lookups
    plan = ora.reorder_plan(shape, idx, off)
    pairs = sorted((int(r), l) for l, r in enumerate(idx) if 0 <= r < shape.num_rows)
    assert plan["any_invalid"] and plan["num_valid"] == len(pairs)
    assert [p[1] for p in pairs] == plan["perm"].tolist()
    assert [p[0] for p in pairs] == plan["sorted_row"].tolist()
    uniq = sorted(set(p[0] for p in pairs))
    assert plan["uniq_row"].tolist() == uniq
    assert np.all(np.diff(plan["uniq_row"]) > 0)
    for l, r in enumerate(idx):
        if 0 <= r < shape.num_rows:
            assert plan["uniq_row"][plan["lookup2row"][l]] == r
        else:
            assert plan["lookup2row"][l] == -1
    seg = plan["row_seg"]
    assert seg[0] == 0 and seg[-1] == len(pairs)
    for u in range(len(uniq)):
        assert np.all(plan["sorted_row"][seg[u]:seg[u + 1]] == uniq[u])
    bag = np.repeat(np.arange(len(off) - 1), np.diff(off))
    assert np.array_equal(plan["bag_of_sorted"], bag[plan["perm"]])
    prefs = sorted(set(r // shape.n[2] for r in uniq))
    assert plan["uniq_pref"].tolist() == prefs
    for q in range(len(prefs)):
        rows = plan["uniq_row"][plan["pref_seg"][q]:plan["pref_seg"][q + 1]]
        assert len(rows) > 0 and np.all(rows // shape.n[2] == prefs[q])
    assert np.array_equal(plan["uniq_pref"][plan["row2pref"]], plan["uniq_row"] // shape.n[2])


def test_reorder_plan_with_remap(ora):
    shape, cores, idx, off, _ = wl.small_random_problem(52, num_bags=20)
    remap = np.random.default_rng(3).permutation(shape.num_rows)
    plan = ora.reorder_plan(shape, idx, off, remap=remap)
    assert np.array_equal(plan["uniq_row"], np.unique(remap[idx]))
    assert np.array_equal(plan["uniq_row"][plan["lookup2row"]], remap[idx])


# ------------------------------------------- dedup mode against definition mode
@pytest.mark.parametrize("cfg_id", [1, 2])
def test_dedup_mode_matches_definition_mode_at_config_sizes(ora, cfg_id):
    cfg = wl.get_config(cfg_id)
    shape, cores = cfg.tables[0], wl.make_cores(cfg, 0)
    idx, off = wl.make_batch(cfg, 0)
    grad = wl.make_grad(cfg, 0)
    a = ora.forward(shape, cores, idx, off)
    b = ora.forward(shape, cores, idx, off, dedup=True)
    np.testing.assert_allclose(b, a, rtol=1e-6, atol=1e-9)
    ga = ora.backward(shape, cores, idx, off, grad)
    gb = ora.backward(shape, cores, idx, off, grad, dedup=True)
    for k in range(3):
        scale = np.abs(ga[k]).max()
        assert np.abs(ga[k] - gb[k]).max() <= 1e-6 * scale
    # Euler identity at this size too
    l0 = float((a.astype(np.float64) * grad.reshape(a.shape)).sum())
    for k in range(3):
        assert abs(float(np.dot(ga[k].astype(np.float64), cores[k].astype(np.float64))) - l0) <= 1e-5 * abs(l0) + 1e-6


# ----------------------------------------------------------------- index graph
def test_index_graph_edges_on_a_hand_computed_batch(ora):
    """Four bags over ranks written out by hand.  rank = identity, hot threshold 2 (rows 0..2 -> node 0).
    bag 0 = rows {5, 3, 5, 9}  -> nodes {3, 1, 7}   pairs (1,3) (1,7) (3,7)
    bag 1 = rows {3, 9, 1}     -> nodes {1, 7}      pair  (1,7)            (row 1 is hot)
    bag 2 = rows {9}           -> no pair
    bag 3 = rows {3, 5, 9, 4}  -> nodes {1, 3, 7, 2}, max_group 3 keeps {1, 2, 3}: (1,2) (1,3) (2,3)"""
    idx = np.array([5, 3, 5, 9, 3, 9, 1, 9, 3, 5, 9, 4], np.int64)
    off = np.array([0, 4, 7, 8, 12], np.int64)
    got = ora.index_graph_edges(idx, off, np.arange(10), hot_thresh=2, max_group=3)
    assert got == {(1, 3): 2, (1, 7): 2, (3, 7): 1, (1, 2): 1, (2, 3): 1}
    # without the group limit bag 3 pairs all four of its nodes
    got = ora.index_graph_edges(idx, off, np.arange(10), hot_thresh=2, max_group=64)
    assert got == {(1, 3): 2, (1, 7): 3, (3, 7): 2, (1, 2): 1, (2, 3): 1, (2, 7): 1}
    # total weight = sum over bags of C(distinct kept nodes, 2)
    assert sum(got.values()) == 3 + 1 + 0 + 6
