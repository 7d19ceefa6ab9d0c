"""GPU parity at the sizes of configs 3-5 (through the C ABI, same launch configuration as
bench.py): full-size outputs against the oracle's dedup mode (itself pinned to definition mode
in the CPU suite), definition mode on a reduced batch, Euler's identity on the remaining tables,
and the two-stream pipeline against the sequential order."""
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


def gpu_step(g, table, idx, off, grad, naive=False):
    import paper_2507_14668_amd as tt
    d_idx, d_off = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64)
    plan = None if naive else tt.tt_index_reorder(table, d_idx, d_off)
    out = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    dg = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, g.to_dev(grad, torch.float32))
    torch.cuda.synchronize()
    if plan is not None:
        assert tt.tt_plan_status(plan) == 0
    return plan, out, dg


def fused_update_check(g, shape, cores, plan, idx, off, grad, lr, updated_table, ref_new, what):
    """Fused backward + update (Section III-F) on fresh cores: against the oracle's updated cores
    and bitwise against backward followed by update."""
    import paper_2507_14668_amd as tt
    fresh = g.gpu_table(shape, cores)
    tt.tt_emb_bag_backward_sgd(fresh, plan, g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64),
                               g.to_dev(grad, torch.float32), lr)
    torch.cuda.synchronize()
    g.assert_grads_close(shape, fresh.cores, ref_new, what="%s fused updated G" % what)
    for k in range(3):
        assert torch.equal(fresh.cores[k], updated_table.cores[k]), "%s: fused update differs (core %d)" % (what, k)


def euler_check(shape, cores, out, dg, grad):
    """<dG_k, G_k> = sum_b <out_b, g_b> for k = 1,2,3 (each row is linear in every core)."""
    o = out.double().cpu().numpy()
    loss = float((o * grad.reshape(o.shape).astype(np.float64)).sum())
    scale = float(np.abs(o * grad.reshape(o.shape)).sum())
    for k in range(3):
        inner = float(np.dot(dg[k].double().cpu().numpy(), cores[k].astype(np.float64)))
        assert abs(inner - loss) <= 1e-5 * scale, (k, inner, loss, scale)


@pytest.mark.parametrize("permute", [False, True])
def test_config3_4_reduced_batch_definition_mode(g, ora, permute):
    print("case cfg3/4 reduced permute=%s" % permute, flush=True)
    cfg = wl.get_config(4)
    shape, cores = cfg.tables[0], wl.make_cores(cfg, 0)
    idx, off = wl.make_batch(cfg, 0, permute_rows=permute, num_bags=1024)
    grad = wl.make_grad(cfg, 0, num_bags=1024)
    table = g.gpu_table(shape, cores)
    ref_out = ora.forward(shape, cores, idx, off)
    ref_dg = ora.backward(shape, cores, idx, off, grad)
    for naive in (False, True):
        _, out, dg = gpu_step(g, table, idx, off, grad, naive=naive)
        g.assert_close_rows(out.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "cfg3 forward naive=%s" % naive)
        g.assert_grads_close(shape, dg, ref_dg, what="cfg4 dG naive=%s" % naive)


def full_table_check(g, ora, cfg, tab, what, permute=None, naive=False):
    """One table at its full batch size, in bench.py's launch configuration: plan bit for bit against
    the integer oracle; complete outputs, gradients, updated cores and the fused update against the
    oracle's dedup mode (itself pinned to definition mode in the CPU suite); Euler's identity."""
    import paper_2507_14668_amd as tt
    shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
    idx, off = wl.make_batch(cfg, tab, permute_rows=permute)
    grad = wl.make_grad(cfg, tab)
    table = g.gpu_table(shape, cores)
    plan, out, dg = gpu_step(g, table, idx, off, grad)
    print("case %s table %d rows=%d n=%s nnz=%d counts=%s" % (what, tab, shape.num_rows, shape.n, len(idx), plan.counts()[0]),
          flush=True)
    g.assert_plan_equals_oracle(ora, shape, plan, idx, off)
    ref_out = ora.forward(shape, cores, idx, off, dedup=True)
    g.assert_close_rows(out.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "forward")
    out_s = tt.tt_emb_bag_forward_sample(table, plan, g.to_dev(off, torch.int64))
    g.assert_close_rows(out_s.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "forward sample-level")
    ref_dg = ora.backward(shape, cores, idx, off, grad, dedup=True, max_threads_=8)
    g.assert_grads_close(shape, dg, ref_dg, what="dG")
    euler_check(shape, cores, out, dg, grad)
    if naive:  # naive arms at full size: forward against the oracle, backward (atomics) against the oracle
        _, out_n, dg_n = gpu_step(g, table, idx, off, grad, naive=True)
        g.assert_close_rows(out_n.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "forward naive")
        g.assert_grads_close(shape, dg_n, ref_dg, what="dG naive")
    ref_new = ora.sgd(cores, ref_dg, cfg.lr)
    tt.tt_core_sgd_update(table, plan, dg, cfg.lr)
    torch.cuda.synchronize()
    g.assert_grads_close(shape, table.cores, ref_new, what="updated G")
    fused_update_check(g, shape, cores, plan, idx, off, grad, cfg.lr, table, ref_new, what)
    g.report_worst("%s table %d " % (what, tab))


@pytest.mark.parametrize("tab", range(8))
def test_config3_4_full_size(g, ora, tab):
    """All 8 tables of configs 3/4 (config 3 = the forward part, config 4 = backward + update); the
    naive arms (no plan; per-lookup chain, float atomics) on the first and the last table."""
    full_table_check(g, ora, wl.get_config(4), tab, "cfg3/4", naive=tab in (0, 7))


def test_config3_4_full_size_permuted_rows(g, ora):
    """The permuted-row variant (Zipf rank -> random row: three times as many distinct prefixes)."""
    full_table_check(g, ora, wl.get_config(4), 1, "cfg3/4 permuted", permute=True)


def cfg5_tables():
    cfg = wl.get_config(5)
    rows = [t.num_rows for t in cfg.tables]
    order = np.argsort(rows)
    return cfg, [int(order[0]), int(order[len(order) // 2]), int(order[-1])]


@pytest.mark.parametrize("tab", range(26))
def test_config5_full_size(g, ora, tab):
    """Every one of the 26 tables bench.py times (row counts 1e3 .. 4e7: every backward split factor
    the benchmark uses, one and two rounds of workgroups, both radix-sort launch structures)."""
    full_table_check(g, ora, wl.get_config(5), tab, "cfg5")


def test_config5_full_size_permuted_rows_largest_table(g, ora):
    cfg, tabs = cfg5_tables()
    full_table_check(g, ora, cfg, tabs[-1], "cfg5 permuted", permute=True)


def test_config5_definition_mode_sample_of_bags(g, ora):
    """Outputs of sampled bags recomputed one by one with the definition-mode oracle."""
    import paper_2507_14668_amd as tt
    cfg, tabs = cfg5_tables()
    tab = tabs[-1]
    shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
    idx, off = wl.make_batch(cfg, tab)
    table = g.gpu_table(shape, cores)
    d_idx, d_off = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64)
    plan = tt.tt_index_reorder(table, d_idx, d_off)
    out = tt.tt_emb_bag_forward(table, plan, d_idx, d_off).cpu().numpy()
    pick = np.random.default_rng(0).choice(cfg.batch, size=512, replace=False)
    sub_idx = np.concatenate([idx[off[b]:off[b + 1]] for b in pick])
    sub_off = np.concatenate([[0], np.cumsum([off[b + 1] - off[b] for b in pick])]).astype(np.int64)
    ref = ora.forward(shape, cores, sub_idx, sub_off)
    g.assert_close_rows(out[pick], ref, g.FWD_RTOL, shape.dim, "cfg5 sampled bags")


def test_two_stream_pipeline_equals_sequential(g):
    """Reorder of batch b+1 on a second stream while batch b runs forward/backward/update on the
    first: results must equal the sequential order bit for bit."""
    import paper_2507_14668_amd as tt
    cfg, tabs = cfg5_tables()
    tabs = tabs[:2]
    nbatch, nb = 4, 8192
    data = {}
    for tab in tabs:
        shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
        data[tab] = dict(shape=shape, cores=cores,
                         batches=[wl.make_batch(cfg, tab, batch=b, num_bags=nb) for b in range(nbatch)],
                         grads=[wl.make_grad(cfg, tab, batch=b, num_bags=nb) for b in range(nbatch)])

    def run(pipelined):
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        res = {}
        for tab in tabs:
            d = data[tab]
            table = g.gpu_table(d["shape"], d["cores"])
            dev = [(g.to_dev(i, torch.int64), g.to_dev(o, torch.int64)) for i, o in d["batches"]]
            grads = [g.to_dev(x, torch.float32) for x in d["grads"]]
            ws = [tt.alloc_workspace(table, dev[0][0].numel(), nb) for _ in range(2)]
            dcores = table.core_grads_like()
            torch.cuda.synchronize()
            ready = [torch.cuda.Event(), torch.cuda.Event()]
            free = [torch.cuda.Event(), torch.cuda.Event()]
            outs = []
            rs = s2 if pipelined else s1
            plans = [None, None]
            plans[0] = tt.tt_index_reorder(table, dev[0][0], dev[0][1], workspace=ws[0], stream=rs)
            ready[0].record(rs)
            for b in range(nbatch):
                cur, nxt = b % 2, (b + 1) % 2
                if b + 1 < nbatch:
                    if b >= 1:
                        rs.wait_event(free[nxt])
                    plans[nxt] = tt.tt_index_reorder(table, dev[b + 1][0], dev[b + 1][1], workspace=ws[nxt], stream=rs)
                    ready[nxt].record(rs)
                s1.wait_event(ready[cur])
                out = tt.tt_emb_bag_forward(table, plans[cur], dev[b][0], dev[b][1], stream=s1)
                tt.tt_emb_bag_backward(table, plans[cur], dev[b][0], dev[b][1], grads[b], dcores=dcores, stream=s1)
                tt.tt_core_sgd_update(table, plans[cur], dcores, cfg.lr, stream=s1)
                free[cur].record(s1)
                outs.append(out)
            torch.cuda.synchronize()
            res[tab] = ([o.clone() for o in outs], [c.clone() for c in table.cores])
        return res

    seq, pipe = run(False), run(True)
    for tab in tabs:
        for a, b in zip(seq[tab][0], pipe[tab][0]):
            assert torch.equal(a, b)
        for a, b in zip(seq[tab][1], pipe[tab][1]):
            assert torch.equal(a, b)


def test_hip_graph_replay_equals_eager(g):
    """One step (reorder of the next batch on a second stream || forward + fused backward/update
    of the current batch) captured as a HIP graph and replayed: after every replay, with eager work
    and a synchronisation in between, outputs and cores must equal the eager sequence bit for bit.
    The library records only kernel launches into a capture (no allocation, no memset)."""
    import paper_2507_14668_amd as tt
    cfg, tabs = cfg5_tables()
    tab = tabs[1]
    shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
    nb, nbatch, rounds = 4096, 2, 3
    dev = []
    for b in range(nbatch):
        idx, off = wl.make_batch(cfg, tab, batch=b, num_bags=nb)
        dev.append((g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64),
                    g.to_dev(wl.make_grad(cfg, tab, batch=b, num_bags=nb), torch.float32)))
    print("case hip graph replay table %d" % tab, flush=True)

    def eager():
        table = g.gpu_table(shape, cores)
        outs = []
        for r in range(rounds * nbatch):
            i, o, gr = dev[r % nbatch]
            plan = tt.tt_index_reorder(table, i, o)
            outs.append(tt.tt_emb_bag_forward(table, plan, i, o).clone())
            tt.tt_emb_bag_backward_sgd(table, plan, i, o, gr, cfg.lr)
        torch.cuda.synchronize()
        return outs, table

    ref_outs, ref_table = eager()

    table = g.gpu_table(shape, cores)
    ws = [tt.alloc_workspace(table, dev[0][0].numel(), nb) for _ in range(2)]
    out = torch.empty((nb, shape.dim), dtype=torch.float32, device="cuda")
    s1, s2, cap = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    plans = [tt.tt_index_reorder(table, dev[0][0], dev[0][1], workspace=ws[0]), None]
    torch.cuda.synchronize()
    graphs = []
    for b in range(nbatch):  # graph b: reorder(batch b+1) on s2 || forward/backward/update(batch b) on s1
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph, stream=cap):
            s1.wait_stream(cap)
            s2.wait_stream(cap)
            nxt = (b + 1) % nbatch
            plans[nxt % 2] = tt.tt_index_reorder(table, dev[nxt][0], dev[nxt][1], workspace=ws[nxt % 2], stream=s2)
            i, o, gr = dev[b]
            tt.tt_emb_bag_forward(table, plans[b % 2], i, o, out=out, stream=s1)
            tt.tt_emb_bag_backward_sgd(table, plans[b % 2], i, o, gr, cfg.lr, stream=s1)
            cap.wait_stream(s1)
            cap.wait_stream(s2)
        graphs.append(gph)
    scratch = torch.zeros(1 << 20, device="cuda")
    for r in range(rounds * nbatch):
        graphs[r % nbatch].replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_outs[r]), "forward of replay %d differs from the eager step" % r
        scratch.add_(1.0)  # the program's own eager work between replays
        torch.cuda.synchronize()
    for k in range(3):
        assert torch.equal(table.cores[k], ref_table.cores[k]), "core %d after the replays differs" % k


@pytest.mark.skip(reason="batched entry points are switched off (TT_ERR_UNAVAILABLE): their first GPU run "
                         "ended in a memory fault whose cause has not been found; the case must not run on "
                         "the GPU again until it is")
@pytest.mark.parametrize("kind", ["mfma", "plain"])
def test_batched_calls_equal_single_table_calls(g, kind):
    """One launch per kernel for several tables (different row factors, same d and ranks) must give
    bit-for-bit the results of the single-table calls, for the planned and the naive arms."""
    import paper_2507_14668_amd as tt
    if kind == "mfma":
        cfg, tabs = cfg5_tables()
        tabs = tabs + [3]
        nb = 4096
        specs = [(cfg.tables[t], wl.make_cores(cfg, t), wl.make_batch(cfg, t, num_bags=nb),
                  wl.make_grad(cfg, t, num_bags=nb)) for t in tabs]
    else:
        specs = []
        for seed, n in [(71, (5, 7, 9)), (72, (11, 3, 4)), (73, (2, 13, 6))]:
            shape, cores, idx, off, grad = wl.small_random_problem(seed, n=n, d=(2, 3, 4), r=(1, 5, 6, 1),
                                                                  num_bags=300, max_len=7)
            specs.append((shape, cores, (idx, off), grad))
    lr = 0.01
    for planned in (True, False):
        print("case batched kind=%s planned=%s" % (kind, planned), flush=True)
        singles, tables_b, idxs, offs, grads = [], [], [], [], []
        for shape, cores, (idx, off), grad in specs:
            table = g.gpu_table(shape, cores)
            d_idx, d_off, d_g = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), g.to_dev(grad, torch.float32)
            plan = tt.tt_index_reorder(table, d_idx, d_off) if planned else None
            out = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
            dg = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, d_g)
            tt.tt_core_sgd_update(table, plan, dg, lr)
            singles.append((out, dg, table.cores))
            tables_b.append(g.gpu_table(shape, cores))
            idxs.append(d_idx); offs.append(d_off); grads.append(d_g)
        T = len(specs)
        desc = tt.alloc_batch_desc(T)
        plans = [None] * T
        if planned:
            ws = [tt.alloc_workspace(tables_b[t], idxs[t].numel(), offs[t].numel() - 1) for t in range(T)]
            plans = tt.tt_index_reorder_batched(tables_b, idxs, offs, ws, desc)
        outs = [torch.empty((offs[t].numel() - 1, tables_b[t].dim), dtype=torch.float32, device="cuda") for t in range(T)]
        dcs = [tables_b[t].core_grads_like() for t in range(T)]
        tt.tt_emb_bag_forward_batched(tables_b, plans, idxs, offs, outs, desc)
        tt.tt_emb_bag_backward_batched(tables_b, plans, idxs, offs, grads, dcs, desc)
        tt.tt_core_sgd_update_batched(tables_b, plans, dcs, lr, desc)
        torch.cuda.synchronize()
        for t in range(T):
            if planned:
                assert tt.tt_plan_status(plans[t]) == 0
                assert torch.equal(outs[t], singles[t][0]), "forward differs for table %d" % t
                for k in range(3):
                    assert torch.equal(dcs[t][k], singles[t][1][k]), "dG%d differs for table %d" % (k + 1, t)
                    assert torch.equal(tables_b[t].cores[k], singles[t][2][k])
            else:  # naive backward uses float atomics: compare to tolerance
                assert torch.equal(outs[t], singles[t][0])
                for k in range(3):
                    ref = singles[t][1][k]
                    assert (dcs[t][k] - ref).abs().max() <= 1e-4 * ref.abs().max() + 1e-30
