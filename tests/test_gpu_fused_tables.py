"""GPU parity of fused tables (several TT tables with equal column factors and ranks stored as one
table, block-diagonal index space): the lookup map bit for bit against numpy, and the fused forward,
backward, update and fused update against the oracle run on every MEMBER table by itself -- the
oracle never sees the fused table, so the claim that a member's row keeps its three slices
(Section III-B index split, Section II-B TT-matrix equation) is what is being tested."""
import numpy as np
import pytest
import torch

import tt_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


def numpy_fuse(members, idx, off, remaps=None):
    """The fused indices and offsets by their definition."""
    N = [sum(n[k] for _, n in members) for k in range(3)]
    o = [0, 0, 0]
    f_idx, f_off, l0 = [], [], 0
    for t, (nr, n) in enumerate(members):
        i = idx[t].astype(np.int64).copy()
        ok = (i >= 0) & (i < nr)
        if remaps is not None and remaps[t] is not None:
            i[ok] = remaps[t][i[ok]]
            ok = (i >= 0) & (i < nr)
        i3, pre = i % n[2], i // n[2]
        i2, i1 = pre % n[1], pre // n[1]
        v = ((o[0] + i1) * N[1] + o[1] + i2) * N[2] + o[2] + i3
        f_idx.append(np.where(ok, v, -1))
        f_off.append(l0 + off[t][:-1])
        l0 += len(i)
        for k in range(3):
            o[k] += n[k]
    f_off.append(np.array([l0], dtype=np.int64))
    return np.concatenate(f_idx).astype(np.int64), np.concatenate(f_off).astype(np.int64)


def make_members(seed, ns, d, r, num_bags, max_len, num_rows=None):
    """Random member tables + one batch each (bags may be empty; a member may have no bags at all)."""
    out = []
    for t, n in enumerate(ns):
        nr = None if num_rows is None else num_rows[t]
        out.append(wl.small_random_problem(seed + t, n=n, d=d, r=r, num_rows=nr, num_bags=num_bags[t], max_len=max_len))
    return out


def run_fused(g, ora, probs, what, lr=0.05, remaps=None):
    import paper_2507_14668_amd as tt
    shapes = [p[0] for p in probs]
    members = [(s.num_rows, s.n) for s in shapes]
    fused = tt.FusedTables(members, shapes[0].d, shapes[0].r, cores=[p[1] for p in probs])
    d_idx = [g.to_dev(p[2], torch.int64) for p in probs]
    d_off = [g.to_dev(p[3], torch.int64) for p in probs]
    d_rm = None if remaps is None else [None if m is None else g.to_dev(m, torch.int64) for m in remaps]
    f_idx, f_off = fused.fuse_lookups(d_idx, d_off, remaps=d_rm)
    ref_idx, ref_off = numpy_fuse(members, [p[2] for p in probs], [p[3] for p in probs], remaps)
    assert np.array_equal(f_idx.cpu().numpy(), ref_idx), "%s: fused indices" % what
    assert np.array_equal(f_off.cpu().numpy(), ref_off), "%s: fused offsets" % what
    grad = g.to_dev(np.concatenate([p[4] for p in probs]), torch.float32)
    plan = tt.tt_index_reorder(fused.table, f_idx, f_off)
    out = tt.tt_emb_bag_forward(fused.table, plan, f_idx, f_off)
    dg = tt.tt_emb_bag_backward(fused.table, plan, f_idx, f_off, grad)
    torch.cuda.synchronize()
    assert tt.tt_plan_status(plan) == 0
    # the fused table as the integer oracle sees it: only the plan is compared here
    fshape = wl.TableShape(fused.table.num_rows, fused.n, shapes[0].d, shapes[0].r)
    g.assert_plan_equals_oracle(ora, fshape, plan, ref_idx, ref_off)
    # member by member against the oracle on the member table alone
    ranges = fused.bag_ranges([len(p[3]) - 1 for p in probs])
    refs = []
    for t, (shape, cores, idx, off, gr) in enumerate(probs):
        if remaps is not None and remaps[t] is not None:
            idx = remaps[t][idx]
        b0, b1 = ranges[t]
        if b1 == b0:  # a member without bags: nothing to look up, its gradient slices are exactly zero
            ref_dg = [np.zeros(shape.core_size(k), dtype=np.float32) for k in range(3)]
        else:
            ref_out = ora.forward(shape, cores, idx, off, dedup=True)
            g.assert_close_rows(out[b0:b1].cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "%s member %d forward" % (what, t))
            ref_dg = ora.backward(shape, cores, idx, off, gr, dedup=True)
        got = [fused.member_core(t, k, core=dg[k]).contiguous().view(-1) for k in range(3)]
        g.assert_grads_close(shape, got, ref_dg, what="%s member %d dG" % (what, t))
        refs.append(ora.sgd(cores, ref_dg, lr))
    # fused update on a second copy of the fused table, bitwise against backward followed by update
    again = tt.FusedTables(members, shapes[0].d, shapes[0].r, cores=[p[1] for p in probs])
    tt.tt_emb_bag_backward_sgd(again.table, plan, f_idx, f_off, grad, lr)
    tt.tt_core_sgd_update(fused.table, plan, dg, lr)
    torch.cuda.synchronize()
    for k in range(3):
        assert torch.equal(again.table.cores[k], fused.table.cores[k]), "%s: fused update differs (core %d)" % (what, k)
    for t, p in enumerate(probs):
        got = [again.member_core(t, k).contiguous().view(-1) for k in range(3)]
        g.assert_grads_close(p[0], got, refs[t], what="%s member %d updated G" % (what, t))
    g.report_worst(what + " ")
    return fused, plan


@pytest.mark.parametrize("arm", ["mfma", "plain"])
def test_fused_small_members(g, ora, arm):
    """Members of unequal factors, one padded (fewer rows than its factors span), one with bags that are
    all empty, one with no bags; multi-hot bags; a row bijection on one member."""
    print("case fused small arm=%s" % arm, flush=True)
    if arm == "mfma":
        d, r = (4, 8, 4), (1, 32, 32, 1)
    else:
        d, r = (2, 3, 2), (1, 3, 4, 1)
    ns = [(5, 6, 7), (3, 4, 5), (9, 2, 4), (2, 2, 2), (4, 4, 3)]
    probs = make_members(100, ns, d, r, num_bags=[40, 25, 0, 9, 30], max_len=6, num_rows=[None, 55, None, None, None])
    # member 3: bags, but no lookup at all
    sh3, c3, _, _, g3 = probs[3]
    probs[3] = (sh3, c3, np.zeros(0, dtype=np.int64), np.zeros(10, dtype=np.int64), g3)
    rng = np.random.default_rng(7)
    remaps = [None, rng.permutation(55).astype(np.int64), None, None, None]
    run_fused(g, ora, probs, "fused small %s" % arm, remaps=remaps)


def test_fused_invalid_lookups_and_offsets_are_reported(g, ora):
    """An index outside a member's rows becomes -1 (skipped and reported by the reorder), never a row
    of a neighbouring member; malformed member offsets become -1 as well."""
    import paper_2507_14668_amd as tt
    print("case fused invalid", flush=True)
    probs = make_members(300, [(3, 4, 5), (2, 3, 4)], (2, 3, 2), (1, 3, 4, 1), num_bags=[12, 8], max_len=4,
                         num_rows=[57, None])
    members = [(p[0].num_rows, p[0].n) for p in probs]
    fused = tt.FusedTables(members, probs[0][0].d, probs[0][0].r, cores=[p[1] for p in probs])
    idx = [p[2].copy() for p in probs]
    off = [p[3].copy() for p in probs]
    idx[0][1], idx[0][3], idx[1][0] = 57, -4, 24  # 57..59 are padding rows of member 0; 24 = rows of member 1
    f_idx, f_off = fused.fuse_lookups([g.to_dev(x, torch.int64) for x in idx], [g.to_dev(x, torch.int64) for x in off])
    ref_idx, ref_off = numpy_fuse(members, idx, off)
    assert np.array_equal(f_idx.cpu().numpy(), ref_idx) and np.array_equal(f_off.cpu().numpy(), ref_off)
    assert (ref_idx == -1).sum() == 3
    plan = tt.tt_index_reorder(fused.table, f_idx, f_off)
    out = tt.tt_emb_bag_forward(fused.table, plan, f_idx, f_off)
    assert tt.tt_plan_status(plan) != 0
    ranges = fused.bag_ranges([12, 8])
    for t, (shape, cores, _, _, _) in enumerate(probs):  # the invalid lookups contribute nothing
        kept, off_v = [], [0]
        for b in range(len(off[t]) - 1):
            seg = idx[t][off[t][b]:off[t][b + 1]]
            kept.extend(seg[(seg >= 0) & (seg < shape.num_rows)])
            off_v.append(len(kept))
        kept, off_v = np.array(kept, dtype=np.int64), np.array(off_v, dtype=np.int64)
        ref = ora.forward(shape, cores, kept, off_v, dedup=True)
        g.assert_close_rows(out[ranges[t][0]:ranges[t][1]].cpu().numpy(), ref, g.FWD_RTOL, shape.dim, "fused invalid member %d" % t)
    # malformed offsets of member 1: first one not 0, one beyond nnz, last one short of nnz
    bad = off[1].copy()
    bad[0], bad[3], bad[-1] = 1, len(idx[1]) + 5, len(idx[1]) - 1
    _, f_off = fused.fuse_lookups([g.to_dev(x, torch.int64) for x in idx], [g.to_dev(off[0], torch.int64), g.to_dev(bad, torch.int64)])
    got = f_off.cpu().numpy()
    assert got[12] == -1 and got[12 + 3] == -1 and got[12 + 7] == -1 and got[-1] == len(idx[0]) + len(idx[1])
    assert np.array_equal(got[:12], off[0][:-1])
    plan = tt.tt_index_reorder(fused.table, f_idx, f_off)
    tt.tt_emb_bag_forward(fused.table, plan, f_idx, f_off)  # clamped inside the kernels: no fault, and reported
    assert tt.tt_plan_status(plan) != 0


@pytest.mark.parametrize("group", range(4))
def test_config5_fused_full_size(g, ora, group):
    """Config 5 as bench.py runs it: the 26 tables dealt to four fused tables, full batch, every member
    against the oracle."""
    import paper_2507_14668_amd as tt
    cfg = wl.get_config(5)
    parts = tt.fusion_groups([(s.num_rows, s.n) for s in cfg.tables], groups=4)
    members = parts[group]
    print("case cfg5 fused group %d members %s" % (group, members), flush=True)
    probs = []
    for t in members:
        idx, off = wl.make_batch(cfg, t)
        probs.append((cfg.tables[t], wl.make_cores(cfg, t), idx, off, wl.make_grad(cfg, t)))
    run_fused(g, ora, probs, "cfg5 fused group %d" % group, lr=cfg.lr)


def test_config4_two_tables_fused_full_size(g, ora):
    """Multi-hot bags at full size: two tables of config 4 as one."""
    cfg = wl.get_config(4)
    probs = []
    for t in (2, 5):
        idx, off = wl.make_batch(cfg, t)
        probs.append((cfg.tables[t], wl.make_cores(cfg, t), idx, off, wl.make_grad(cfg, t)))
    print("case cfg4 fused tables 2+5", flush=True)
    run_fused(g, ora, probs, "cfg4 fused", lr=cfg.lr)


def test_fused_two_stream_pipeline_equals_sequential(g):
    """The step as bench.py runs it: the lookup map and the reorder of batch b+1 on a second stream
    (two plan buffers, two pairs of fused index buffers) while batch b computes -- bitwise equal to
    running everything on one stream."""
    import paper_2507_14668_amd as tt
    print("case fused pipeline", flush=True)
    cfg = wl.get_config(5)
    members, nb, nbatch = [0, 7, 13, 23], 4096, 5
    shapes = [cfg.tables[t] for t in members]
    host = [[wl.make_batch(cfg, t, batch=b, num_bags=nb) for t in members] for b in range(nbatch)]
    dev = [[(g.to_dev(i, torch.int64), g.to_dev(o, torch.int64)) for i, o in hb] for hb in host]
    grads = [g.to_dev(np.concatenate([wl.make_grad(cfg, t, batch=b, num_bags=nb) for t in members]), torch.float32)
             for b in range(nbatch)]

    def run(pipelined):
        fused = tt.FusedTables([(s.num_rows, s.n) for s in shapes], shapes[0].d, shapes[0].r,
                               cores=[wl.make_cores(cfg, t) for t in members])
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        rs = s2 if pipelined else s1
        nnz, bags = nb * len(members), nb * len(members)
        ws = [tt.alloc_workspace(fused.table, nnz, bags) for _ in range(2)]
        fbuf = [(torch.empty(nnz, dtype=torch.int64, device="cuda"), torch.empty(bags + 1, dtype=torch.int64, device="cuda"))
                for _ in range(2)]
        ready = [torch.cuda.Event(), torch.cuda.Event()]
        free = [torch.cuda.Event(), torch.cuda.Event()]
        torch.cuda.synchronize()

        def plan_of(b, buf):
            fi, fo = fused.fuse_lookups([x[0] for x in dev[b]], [x[1] for x in dev[b]], out=fbuf[buf], stream=rs)
            p = tt.tt_index_reorder(fused.table, fi, fo, workspace=ws[buf], stream=rs)
            ready[buf].record(rs)
            return p

        plans, outs = [plan_of(0, 0), None], []
        for b in range(nbatch):
            cur, nxt = b % 2, (b + 1) % 2
            if b + 1 < nbatch:
                if b >= 1:
                    rs.wait_event(free[nxt])
                plans[nxt] = plan_of(b + 1, nxt)
            s1.wait_event(ready[cur])
            outs.append(tt.tt_emb_bag_forward(fused.table, plans[cur], fbuf[cur][0], fbuf[cur][1], stream=s1))
            tt.tt_emb_bag_backward_sgd(fused.table, plans[cur], fbuf[cur][0], fbuf[cur][1], grads[b], cfg.lr, stream=s1)
            free[cur].record(s1)
        torch.cuda.synchronize()
        return [o.clone() for o in outs], [c.clone() for c in fused.table.cores]

    seq, pipe = run(False), run(True)
    for a, b in zip(seq[0] + seq[1], pipe[0] + pipe[1]):
        assert torch.equal(a, b)


def test_fused_seeded_random_members(g, ora):
    """Twelve seeded random fused tables: two to seven members with random row factors, row counts
    (some padded), batch sizes and bag lengths, on both kernel families."""
    rng = np.random.default_rng(20251)
    for case in range(12):
        mfma = case % 2 == 0
        d, r = ((4, 8, 4), (1, 32, 32, 1) if case % 4 == 0 else (1, 64, 64, 1)) if mfma else ((2, 3, 2), (1, int(rng.integers(2, 6)), int(rng.integers(2, 6)), 1))
        members = int(rng.integers(2, 8))
        ns = [tuple(int(x) for x in rng.integers(1, 13, size=3)) for _ in range(members)]
        rows = [int(rng.integers(max(1, n[0] * n[1] * n[2] - n[2] + 1), n[0] * n[1] * n[2] + 1)) for n in ns]
        bags = [int(rng.integers(0, 70)) for _ in range(members)]
        print("case fused random %d d=%s r=%s ns=%s rows=%s bags=%s" % (case, d, r, ns, rows, bags), flush=True)
        probs = make_members(7000 + 10 * case, ns, d, r, num_bags=bags, max_len=int(rng.integers(1, 9)), num_rows=rows)
        run_fused(g, ora, probs, "fused random %d" % case)


def test_fuse_lookups_more_lookups_than_one_grid_pass(g):
    """A member with 1.3 million lookups (the map's grid is capped and strides) beside a small one and an
    empty one: the map bit for bit against numpy."""
    import paper_2507_14668_amd as tt
    print("case fuse_lookups 1.3M", flush=True)
    rng = np.random.default_rng(5)
    members = [(90000, (45, 50, 40)), (60, (3, 4, 5)), (1000, (10, 10, 10))]
    lens = [rng.integers(0, 6, size=520_000), np.zeros(0, dtype=np.int64), rng.integers(0, 3, size=77)]
    idx, off = [], []
    for (nr, _), ln in zip(members, lens):
        o = np.zeros(len(ln) + 1, dtype=np.int64)
        np.cumsum(ln, out=o[1:])
        off.append(o)
        idx.append(rng.integers(-2, nr + 2, size=int(o[-1]), dtype=np.int64))  # a few invalid ones on both sides
    assert len(idx[0]) > 1_200_000
    layout = tt.FusedLayout(members)
    f_idx, f_off = layout.fuse_lookups([g.to_dev(x, torch.int64) for x in idx], [g.to_dev(x, torch.int64) for x in off])
    ref_idx, ref_off = numpy_fuse(members, idx, off)
    assert np.array_equal(f_idx.cpu().numpy(), ref_idx) and np.array_equal(f_off.cpu().numpy(), ref_off)
    assert (ref_idx == -1).sum() > 10
