#!/usr/bin/env python3
"""Throughput of the TT embedding-bag hot path on one MI355X.

One step = one pass of the whole hot path over one batch of every table of the workload:
index reorder (for the NEXT batch, on a second stream) || forward + backward + core update
(for the current batch).  Inputs are synthetic (tt_workloads.py), resident in HBM before the
timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0      # MI355X HBM3E, published
PEAK_FP32_TFLOPS = 157.3   # MI355X fp32 (vector or matrix), published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--arm", default="plan", choices=["plan", "naive", "sample", "bf16"],
                    help="plan: batch-level reuse; naive: no plan; sample: plan + sample-level reuse forward; "
                         "bf16: plan + forward on bf16 copies of the cores (both forward-only workloads)")
    ap.add_argument("--no-overlap", action="store_true", help="reorder on the compute stream")
    ap.add_argument("--permute", action="store_true", help="seeded random row permutation of the Zipf ranks")
    ap.add_argument("--bijection", action="store_true",
                    help="build the offline index bijection (frequency order; the synthetic batches have no "
                         "co-occurrence structure) from the batches and pass it to the reorder as `remap`")
    ap.add_argument("--batches", type=int, default=8, help="distinct batches cycled through")
    ap.add_argument("--tables", type=int, default=0, help="use only the first T tables (0 = all)")
    ap.add_argument("--streams", type=int, default=-1,
                    help="tables are dealt round-robin to this many (compute, reorder) stream pairs "
                         "(-1: 8, or 2 when the tables are fused)")
    ap.add_argument("--fuse", type=int, default=-1,
                    help="deal the tables to this many FUSED tables (tables with equal column factors and ranks "
                         "stored as one table; the map of the members' lookups, tt_fuse_lookups, runs inside the "
                         "timed step, in front of the reorder).  0: one table per call; -1: 4 for cfg5, 0 otherwise")
    ap.add_argument("--host-threads", type=int, default=4,
                    help="host threads that enqueue the stream pairs of a step in parallel")
    ap.add_argument("--graph", action="store_true",
                    help="capture each step of the timed region (all tables, all stream pairs) in a HIP "
                         "graph and replay it, so that the host enqueues one graph instead of ~1000 kernels")
    ap.add_argument("--separate-update", action="store_true",
                    help="backward writes the core gradients and a separate call applies them "
                         "(default: the fused backward+update call)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", dest="other_configs", action="store_false",
                    help="with the default workload, skip the shorter runs of configs 3 and 4 (plan and naive "
                         "arms) that are reported as `other_configs` in the same line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of known size (256 MiB read + 256 MiB written, five "
                         "times): the reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--prof-kernel", default="auto",
                    choices=["auto", "fwd_contract", "bwd_contract", "bag_sum", "grad_merge", "p12_fill", "bag_chains"],
                    help="kernel bracketed with HIP events for the roofline (auto = the dominant one)")
    return ap.parse_args()


def measure(args, workload, arm, steps, warmup, batches, prof_kernels, streams, fuse=0):
    """One workload and arm: `warmup` + `steps` steps on `streams` stream pairs -> throughput; then, for
    every kernel in `prof_kernels` (planned arm), the same steps on ONE stream pair with that kernel
    bracketed by HIP events -> its roofline entry.  Returns the result dict of the JSON line (the first
    entry of prof_kernels is `roofline`, all of them are in `kernel_rooflines`)."""
    import numpy as np
    import torch

    import paper_2507_14668_amd as tt
    import tt_workloads as wl
    from paper_2507_14668_amd import binding  # noqa: F401

    cfg_id = int(workload[3:])
    cfg = wl.get_config(cfg_id)
    do_bwd = cfg_id != 3
    ntab = len(cfg.tables) if args.tables <= 0 else min(args.tables, len(cfg.tables))
    nbatch = max(2, batches + (batches % 2))  # even, so batch b always uses plan buffer b%2

    # ---- inputs, resident in HBM ------------------------------------------------------------
    t_gen = time.time()
    tabs = []
    for t in range(ntab):
        shape = cfg.tables[t]
        table = tt.Table.from_numpy(shape, wl.make_cores(cfg, t))
        batches = []
        host = [wl.make_batch(cfg, t, batch=b, permute_rows=True if args.permute else None) for b in range(nbatch)]
        remap = None
        if args.bijection:
            from paper_2507_14668_amd.bijection import build_index_bijection
            # learned from OTHER batches of the same distribution than the ones that are timed
            sample = [wl.make_batch(cfg, t, batch=nbatch + b, permute_rows=True if args.permute else None)
                      for b in range(nbatch)]
            remap = build_index_bijection(sample, shape.num_rows, hot_ratio=1.0)
        for b in range(nbatch):
            idx, off = host[b]
            grad = wl.make_grad(cfg, t, batch=b)
            seen = idx if remap is None else remap[idx]  # the rows the kernels actually touch
            batches.append(dict(idx=torch.from_numpy(idx).cuda(), off=torch.from_numpy(off).cuda(),
                                grad=torch.from_numpy(grad).cuda(), nnz=len(idx),
                                # workload statistics used only to count algorithmic work
                                u_r=int(np.unique(seen).size), u_p=int(np.unique(seen // shape.n[2]).size),
                                # (bag, prefix) groups: second-stage products of the sample-level route
                                groups=int(np.unique(np.repeat(np.arange(len(off) - 1, dtype=np.int64), np.diff(off)) *
                                                     (shape.n[0] * shape.n[1]) + seen // shape.n[2]).size)
                                if arm == "sample" else None))
        max_nnz = max(x["nnz"] for x in batches)
        ws = [tt.alloc_workspace(table, max_nnz, cfg.batch) for _ in range(2)] if arm != "naive" else None
        reuse = (torch.empty(tt.tt_reuse_buffer_bytes(table, max_nnz), dtype=torch.uint8, device="cuda")
                 if arm == "sample" else None)
        tabs.append(dict(shape=shape, table=table, batches=batches, ws=ws, plans=[None, None], reuse=reuse,
                         bf16=tt.tt_cores_to_bf16(table) if arm == "bf16" else None,
                         remap=None if remap is None else torch.from_numpy(remap).cuda(),
                         out=torch.empty((cfg.batch, shape.dim), dtype=torch.float32, device="cuda"),
                         dcores=table.core_grads_like()))
    planned = arm != "naive"
    ntab_members = ntab
    for T in tabs:
        T["bags"] = cfg.batch
    if fuse > 0 and planned:
        # Fused tables: the members' cores side by side in one table; the members' index and offset
        # tensors stay the inputs of the step, their map into the fused table is part of the step.
        sh0 = cfg.tables[0]
        parts = tt.fusion_groups([(T["shape"].num_rows, T["shape"].n) for T in tabs], groups=fuse)
        ftabs = []
        for members in parts:
            M = [tabs[t] for t in members]
            fused = tt.FusedTables([(T["shape"].num_rows, T["shape"].n) for T in M], sh0.d, sh0.r,
                                   cores=[T["table"].cores for T in M])
            fb = []
            for b in range(nbatch):
                xs = [T["batches"][b] for T in M]
                fb.append(dict(m_idx=[x["idx"] for x in xs], m_off=[x["off"] for x in xs],
                               grad=torch.cat([x["grad"] for x in xs]), nnz=sum(x["nnz"] for x in xs),
                               u_r=sum(x["u_r"] for x in xs), u_p=sum(x["u_p"] for x in xs),
                               groups=sum(x["groups"] for x in xs) if arm == "sample" else None))
            max_nnz, bags = max(x["nnz"] for x in fb), cfg.batch * len(M)
            ftabs.append(dict(shape=wl.TableShape(fused.table.num_rows, fused.n, sh0.d, sh0.r), table=fused.table,
                              fused=fused, members=members, batches=fb, plans=[None, None], bags=bags,
                              ws=[tt.alloc_workspace(fused.table, max_nnz, bags) for _ in range(2)],
                              fidx=[torch.empty(max_nnz, dtype=torch.int64, device="cuda") for _ in range(2)],
                              foff=[torch.empty(bags + 1, dtype=torch.int64, device="cuda") for _ in range(2)],
                              m_remaps=[T["remap"] for T in M] if args.bijection else None, remap=None,
                              reuse=(torch.empty(tt.tt_reuse_buffer_bytes(fused.table, max_nnz), dtype=torch.uint8, device="cuda")
                                     if arm == "sample" else None),
                              bf16=tt.tt_cores_to_bf16(fused.table) if arm == "bf16" else None,
                              out=torch.empty((bags, sh0.dim), dtype=torch.float32, device="cuda"),
                              dcores=fused.table.core_grads_like()))
        for T in tabs:
            T["ws"] = T["out"] = T["dcores"] = T["reuse"] = None
        tabs = ftabs
        ntab = len(tabs)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    def make_plan(T, x, buf, stream):
        """The plan of batch x in plan buffer `buf`; a fused table first maps its members' lookups."""
        if "fused" in T:
            idx, off = T["fused"].fuse_lookups(x["m_idx"], x["m_off"], remaps=T["m_remaps"],
                                               out=(T["fidx"][buf][:x["nnz"]], T["foff"][buf]), stream=stream)
            T["lookups"][buf] = (idx, off)
            return tt.tt_index_reorder(T["table"], idx, off, workspace=T["ws"][buf], stream=stream)
        T["lookups"][buf] = (x["idx"], x["off"])
        # workspace sized for the largest batch; the plan is rebuilt for this batch's nnz
        return tt.tt_index_reorder(T["table"], x["idx"], x["off"], remap=T["remap"], workspace=T["ws"][buf], stream=stream)

    for T in tabs:
        T["lookups"] = [None, None]
    if arm in ("sample", "bf16"):
        assert not do_bwd, "the %s arm is a forward: use a forward-only workload (cfg3)" % arm

    def compute_table(T, x, buf, stream):
        """Forward and (with a backward workload) backward + update of batch x of one table."""
        plan = T["plans"][buf] if planned else None
        idx, off = T["lookups"][buf] if planned else (x["idx"], x["off"])
        if arm == "sample":
            tt.tt_emb_bag_forward_sample(T["table"], plan, off, reuse_buffer=T["reuse"], out=T["out"], stream=stream)
        elif arm == "bf16":
            tt.tt_emb_bag_forward_bf16(T["table"], T["bf16"], plan, off, out=T["out"], stream=stream)
        else:
            tt.tt_emb_bag_forward(T["table"], plan, idx, off, out=T["out"], stream=stream)
        if do_bwd and planned and not args.separate_update:
            tt.tt_emb_bag_backward_sgd(T["table"], plan, idx, off, x["grad"], cfg.lr, stream=stream)
        elif do_bwd:
            tt.tt_emb_bag_backward(T["table"], plan, idx, off, x["grad"], dcores=T["dcores"], stream=stream)
            tt.tt_core_sgd_update(T["table"], plan, T["dcores"], cfg.lr, stream=stream)

    prof_kernels = [("bwd_contract" if do_bwd else "fwd_contract") if k == "auto" else k for k in prof_kernels]
    if not planned:
        prof_kernels = []
    profs = {k: tt.Prof(k, (steps + 1) * ntab * 4) for k in prof_kernels}
    cur = {"name": prof_kernels[0] if prof_kernels else None}  # the kernel the next bracketed region selects

    def run_region(ns, warmup, steps, bracket, use_graph=False):
        """`warmup` untimed and `steps` timed steps with `ns` stream pairs: table t computes on
        cs[t % ns] and has the NEXT batch reordered on rs[t % ns] (all default priority).  Tables
        on different pairs run concurrently, which fills the chip when one table's kernels are too
        small to do so.  With `bracket`, the selected kernel of every launch in the timed steps is
        bracketed with HIP events on its launch stream."""
        cs = [torch.cuda.Stream() for _ in range(ns)]
        rs = cs if args.no_overlap else [torch.cuda.Stream() for _ in range(ns)]
        ready = [[torch.cuda.Event(), torch.cuda.Event()] for _ in range(ns)]
        free = [[torch.cuda.Event(), torch.cuda.Event()] for _ in range(ns)]
        groups = [[T for i, T in enumerate(tabs) if i % ns == k] for k in range(ns)]
        timing = [False]
        pool = None
        if args.host_threads > 1 and ns > 1 and not use_graph and not bracket:
            from concurrent.futures import ThreadPoolExecutor
            pool = ThreadPoolExecutor(max_workers=min(args.host_threads, ns))

        def reorder(b, events=True):
            buf = b % 2
            for k in range(ns):
                for T in groups[k]:
                    T["plans"][buf] = make_plan(T, T["batches"][b % nbatch], buf, rs[k])
                    if timing[0]:
                        profs[cur["name"]].attach(T["plans"][buf])
                if events:
                    ready[k][buf].record(rs[k])

        def compute(b, events=True):
            buf = b % 2
            for k in range(ns):
                if planned and events:
                    cs[k].wait_event(ready[k][buf])
                for T in groups[k]:
                    compute_table(T, T["batches"][b % nbatch], buf, cs[k])
                if events:
                    free[k][buf].record(cs[k])

        def step(b):
            """reorder(b+1) on the reorder streams while batch b computes; plan buffer (b+1)%2 was
            last used by the compute of batch b-1."""
            if pool is not None:  # the stream pairs are independent: enqueue them from several threads
                list(pool.map(lambda k: step_pair(b, k), range(ns)))
                return
            if planned:
                for k in range(ns):
                    rs[k].wait_event(free[k][(b + 1) % 2])
                reorder(b + 1)
            compute(b)

        def step_pair(b, k):
            buf, nxt = b % 2, (b + 1) % 2
            if planned:
                rs[k].wait_event(free[k][nxt])
                for T in groups[k]:
                    T["plans"][nxt] = make_plan(T, T["batches"][(b + 1) % nbatch], nxt, rs[k])
                    if timing[0]:
                        profs[cur["name"]].attach(T["plans"][nxt])
                ready[k][nxt].record(rs[k])
                cs[k].wait_event(ready[k][buf])
            for T in groups[k]:
                compute_table(T, T["batches"][b % nbatch], buf, cs[k])
            free[k][buf].record(cs[k])

        def capture(b):
            """One step as a HIP graph: the capture stream forks into every stream pair, reorder(b+1)
            and compute(b) are recorded without cross-step events (consecutive replays on one stream
            are ordered as a whole, and inside a step the two do not depend on each other), and all
            streams join again.  The library allocates nothing and records no memset."""
            g = torch.cuda.CUDAGraph()
            cap = torch.cuda.Stream()
            with torch.cuda.graph(g, stream=cap):
                for st in set(cs) | set(rs):
                    st.wait_stream(cap)
                if planned:
                    reorder(b + 1, events=False)
                compute(b, events=False)
                for st in set(cs) | set(rs):
                    cap.wait_stream(st)
            return g

        graphs = None
        if use_graph:
            assert not bracket, "kernel brackets are HIP events and cannot be replayed from a graph"
            if planned:
                reorder(0)  # one eager step first: module load and launch attributes precede any capture
            step(0)
            torch.cuda.synchronize()
            if planned:
                reorder(0, events=False)
            torch.cuda.synchronize()
            graphs = [capture(i) for i in range(nbatch)]
            replay_stream = torch.cuda.Stream()

            def step(b):  # noqa: F811 - the captured step replaces the eager one
                with torch.cuda.stream(replay_stream):
                    graphs[b % nbatch].replay()

        # prologue: plan of batch 0, both 'free' events recorded so the first waits pass
        torch.cuda.synchronize()
        for k in range(ns):
            free[k][0].record(cs[k])
            free[k][1].record(cs[k])
        if planned and not use_graph:
            reorder(0)
        b = 0
        for _ in range(warmup):
            step(b)
            b += 1
        torch.cuda.synchronize()
        lookups = 0
        prof_name = cur["name"]
        if planned and bracket:
            timing[0] = True
            for T in tabs:
                profs[prof_name].attach(T["plans"][b % 2])
        t0 = time.perf_counter()
        for _ in range(steps):
            step(b)
            lookups += sum(T["batches"][b % nbatch]["nnz"] for T in tabs)
            b += 1
        t_enqueue = time.perf_counter() - t0  # host time spent enqueueing (GPU may still be running)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        res = dict(dt=dt, t_enqueue=t_enqueue, lookups=lookups, last_b=b, roofline=None)
        if planned and bracket:
            kernel_ms, launches = profs[prof_name].collect()
            for T in tabs:  # later regions must not record into the same event pool
                for pl in T["plans"]:
                    if pl is not None:
                        pl.c.prof = None
            first = b - steps
            work = 0.0
            for k in range(steps):
                for T in tabs:
                    work += kernel_work(prof_name, T["shape"], T["batches"][(first + k) % nbatch], T["bags"])
            bound, unit, peak, scale = KERNEL_BOUND[prof_name]
            if launches > 0 and kernel_ms > 0:
                achieved = work / (kernel_ms * 1e-3) / scale
                res["roofline"] = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                                   "frac": achieved / peak, "traffic": read_traffic(workload, prof_name),
                                   "kernel": prof_name, "launches": int(launches),
                                   "avg_launch_us": 1e3 * kernel_ms / launches,
                                   "algorithmic_work_per_launch": work / launches,
                                   "stream_pairs": ns}
        return res

    # Timed region: K steps of the whole job on `--streams` stream pairs -> value.  With more than
    # one pair the kernels of different tables overlap and a bracketed kernel's duration includes
    # contention, so the roofline of the dominant kernel is then taken from a second timed pass of
    # the same K steps on ONE pair, where the bracketed kernel has the chip to itself (this is also
    # the condition under which a rocprofv3 kernel trace, which serialises dispatches, sees it).
    if streams <= 0:
        streams = 2 if ntab != ntab_members else 8
    ns = max(1, min(streams, ntab))
    solo_main = ns == 1 and not args.graph and len(prof_kernels) == 1
    main_region = run_region(ns, warmup, steps, bracket=solo_main and bool(prof_kernels), use_graph=args.graph)
    dt, t_enqueue, lookups, b = main_region["dt"], main_region["t_enqueue"], main_region["lookups"], main_region["last_b"]
    kernel_rooflines = {}
    solo_region = None
    for name in prof_kernels:
        cur["name"] = name
        solo_region = main_region if solo_main else run_region(1, 1, steps, bracket=True)
        r = solo_region["roofline"]
        if r is not None and not solo_main:
            r["measured_in"] = "second timed pass of the same %d steps on 1 stream pair (%.3f ms/step)" % (
                steps, 1e3 * solo_region["dt"] / steps)
        kernel_rooflines[name] = r
    roofline = kernel_rooflines[prof_kernels[0]] if prof_kernels else None

    status_bad = 0
    counts = []
    if planned:
        for T in tabs:
            c, st = T["plans"][((solo_region or main_region)["last_b"] - 1) % 2].counts()
            status_bad |= st != 0
            counts.append(c)
    assert not status_bad, "a plan reported an index/offset error"

    value = lookups / dt
    phases = "reorder||fwd" if not do_bwd else "reorder||fwd+bwd+update"
    if do_bwd and planned and not args.separate_update:
        phases += " (update fused into bwd)"
    result = {
        "metric": "TT embedding lookups/sec fwd+bwd (1 GPU)", "value": value, "unit": "lookups/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": 1e3 * dt / steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d TT tables, D=%d, ranks (1,%d,%d,1), batch %d %s bags per table, "
                               "Zipf(alpha=%g)%s, %s, %s arm" %
                               (workload, ntab_members, cfg.tables[0].dim, cfg.tables[0].r[1], cfg.tables[0].r[2],
                                cfg.batch, "multi-hot" if cfg.multi_hot else "one-hot", cfg.alpha,
                                (" + row permutation" if (args.permute or cfg.permute_rows) else "") +
                                (" + offline index bijection" if args.bijection else ""),
                                phases, arm) + (", tables fused into %d (lookup map inside the step)" % ntab
                                                if ntab != ntab_members else ""),
                   "lookups_per_step": lookups // max(1, steps), "tables": ntab_members,
                   "fused_tables": ntab if ntab != ntab_members else 0,
                   "overlap_second_stream": (not args.no_overlap) and planned, "stream_pairs": ns,
                   "hip_graph_replay": bool(args.graph), "host_enqueue_threads": args.host_threads,
                   "host_enqueue_ms_per_step": round(1e3 * t_enqueue / steps, 3),
                   "input_generation_s": round(t_gen, 1)},
        "roofline": roofline,
        "cpu_baseline": None,
        "kernel_rooflines": {k: v for k, v in kernel_rooflines.items() if v is not None},
    }
    if planned:  # whole-step roofline: algorithmic work of one step against the published peaks
        flops = bytes_ = 0.0
        first = main_region["last_b"] - steps
        for k in range(steps):
            for T in tabs:
                x = T["batches"][(first + k) % nbatch]
                nt = len(T.get("members", [0]))  # every member table brings its own offsets array
                flops += kernel_work("fwd_contract", T["shape"], x, T["bags"]) + x["nnz"] * T["shape"].dim
                bytes_ += 8.0 * x["nnz"] + 8.0 * (T["bags"] + nt) + 4.0 * T["bags"] * T["shape"].dim  # indices, offsets, out
                if do_bwd:
                    flops += kernel_work("bwd_contract", T["shape"], x, T["bags"]) + x["nnz"] * T["shape"].dim
                    bytes_ += 4.0 * T["bags"] * T["shape"].dim  # output gradients
        t_flop, t_hbm = flops / steps / (PEAK_FP32_TFLOPS * 1e12), bytes_ / steps / (PEAK_HBM_GBS * 1e9)
        result["config"]["step_bound_ms"] = {"fp32_mfma": round(1e3 * t_flop, 4), "hbm": round(1e3 * t_hbm, 4),
                                             "frac_of_measured": round(max(t_flop, t_hbm) / (dt / steps), 4)}
    if arm == "sample":
        result["config"]["bag_prefix_groups_batch0"] = int(sum(T["batches"][0]["groups"] for T in tabs))
        result["config"]["lookups_batch0"] = int(sum(T["batches"][0]["nnz"] for T in tabs))
    if counts:
        result["config"]["distinct_rows_last_batch"] = int(sum(c[0] for c in counts))
        result["config"]["distinct_prefixes_last_batch"] = int(sum(c[1] for c in counts))

    for T in tabs:  # release the device memory before the next workload is set up
        T.clear()
    for pr in profs.values():
        pr.close()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return result


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2507_14668_amd as tt
    import tt_workloads as wl
    from paper_2507_14668_amd import binding

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = 64 * 1024 * 1024
        src = torch.arange(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "launches": 5, "bytes_read_per_launch": 4 * n,
                          "bytes_written_per_launch": 4 * n}))
        return
    tt.load_library()
    # the dominant kernel first (-> `roofline`); with the default choice also the other kernels of the step
    headline_kernels = [args.prof_kernel] if args.prof_kernel != "auto" else (
        ["auto", "fwd_contract", "bag_sum", "grad_merge"] if args.arm == "plan" and args.workload != "cfg3" else ["auto"])
    fuse = args.fuse if args.fuse >= 0 else (4 if args.workload == "cfg5" else 0)
    result = measure(args, args.workload, args.arm, args.steps, args.warmup, args.batches, headline_kernels, args.streams,
                     fuse=fuse)
    if args.other_configs and args.workload == "cfg5" and args.arm == "plan":
        # the other configurations the target names, in the same line: two batches each, and few steps for
        # the naive arms (they take tens to hundreds of milliseconds per step)
        other = {}
        for wk, arm_, st_, kern in (("cfg3", "plan", 30, ["fwd_contract", "bag_sum"]), ("cfg3", "naive", 3, []),
                                    ("cfg3", "sample", 30, ["bag_chains", "p12_fill"]),
                                    ("cfg3", "bf16", 30, ["fwd_contract"]),
                                    ("cfg4", "plan", 30, ["bwd_contract", "grad_merge", "fwd_contract", "bag_sum"]),
                                    ("cfg4", "naive", 2, []),
                                    # the headline workload with one call per table instead of fused tables
                                    ("cfg5", "plan_per_table", 20, ["bwd_contract", "fwd_contract"])):
            if arm_ == "plan_per_table":
                r = measure(args, wk, "plan", st_, 3, 2, kern, args.streams, fuse=0)
            else:
                r = measure(args, wk, arm_, st_, 3 if arm_ != "naive" else 1, 2, kern, args.streams)
            entry = {"ms_per_step": r["ms_per_step"], "lookups_per_s": r["value"], "steps": st_,
                     "workload": r["config"]["workload"]}
            for key in ("bag_prefix_groups_batch0", "lookups_batch0", "distinct_rows_last_batch", "distinct_prefixes_last_batch"):
                if key in r["config"]:
                    entry[key] = r["config"][key]
            if "step_bound_ms" in r["config"]:
                entry["step_bound_ms"] = r["config"]["step_bound_ms"]
            if r.get("kernel_rooflines"):
                entry["kernels"] = {k: {x: v[x] for x in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_us")}
                                    for k, v in r["kernel_rooflines"].items()}
            other["%s_%s" % (wk, arm_)] = entry
        result["other_configs"] = other
    kr = result.pop("kernel_rooflines", None) or {}
    if len(kr) > 1:  # the step's other kernels, each from its own timed pass on one stream pair
        result["kernels"] = {k: {x: v[x] for x in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_us")}
                             for k, v in kr.items()}
    cfg = __import__("tt_workloads").get_config(int(args.workload[3:]))
    wl = __import__("tt_workloads")
    np = __import__("numpy")
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, wl, np)
    print(json.dumps(result))


# kernel -> (bound, unit, published MI355X peak in that unit, divisor to that unit)
KERNEL_BOUND = {
    "fwd_contract": ("mfma", "TFLOP/s", PEAK_FP32_TFLOPS, 1e12),
    "bwd_contract": ("mfma", "TFLOP/s", PEAK_FP32_TFLOPS, 1e12),
    "bag_sum": ("hbm", "GB/s", PEAK_HBM_GBS, 1e9),
    "grad_merge": ("hbm", "GB/s", PEAK_HBM_GBS, 1e9),
    "p12_fill": ("mfma", "TFLOP/s", PEAK_FP32_TFLOPS, 1e12),
    "bag_chains": ("hbm", "GB/s", PEAK_HBM_GBS, 1e9),
}


def kernel_work(kernel, shape, batch, num_bags):
    """Algorithmic flops (contractions) or bytes (streaming kernels) of ONE launch: the work the
    method needs after reuse and dedup, not what the implementation happens to move."""
    d1, d2, d3 = shape.d
    r1, r2 = shape.r[1], shape.r[2]
    dim = d1 * d2 * d3
    f12 = 2.0 * d1 * r1 * d2 * r2      # one prefix product G1[i1] x G2[i2]
    f3 = 2.0 * d1 * d2 * r2 * d3       # one row P12 x G3[i3]
    nnz, u_r, u_p = batch["nnz"], batch["u_r"], batch["u_p"]
    if kernel == "fwd_contract":
        return u_p * f12 + u_r * f3
    if kernel == "bwd_contract":
        # per prefix: P12 recomputed (cheaper than 2 x 4 x P12 bytes of traffic), H x G2^T, G1^T x H;
        # per distinct row: P12^T x g and g x G3^T
        return u_p * 3 * f12 + u_r * 2 * f3
    # streaming kernels: COMPULSORY bytes (every distinct row / every bag gradient once), not the bytes
    # gathered: rows and gradients that are read several times come out of the caches
    if kernel == "bag_sum":
        return 4.0 * u_r * dim + 4.0 * num_bags * dim + 4.0 * nnz + 8.0 * (num_bags + 1)
    if kernel == "grad_merge":
        return 4.0 * num_bags * dim + 4.0 * u_r * dim + 8.0 * nnz
    if kernel == "p12_fill":
        return u_p * f12
    if kernel == "bag_chains":  # every prefix product once, every output row once, two index reads per lookup
        return 4.0 * u_p * d1 * d2 * r2 + 4.0 * num_bags * dim + 8.0 * nnz + 8.0 * (num_bags + 1)
    raise ValueError(kernel)


def read_traffic(workload, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), if a summary
    for this workload and kernel has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", "traffic_%s_%s.txt" % (workload, kernel))
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":", 1)[1])
    return None


def cpu_baseline(cfg, wl, np):
    """The oracle (definition mode, forward + backward) timed on a bounded sample of the workload:
    batches of the largest tables, one after the other, until the sample holds at least 10 s of CPU
    work; a batch that would not fit into a budget of about 25 s is cut to a prefix of its bags."""
    from oracle import tt_oracle as ora
    order = list(np.argsort([-t.num_rows for t in cfg.tables]))

    def run(tab, nb):
        shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
        idx, off = wl.make_batch(cfg, tab, num_bags=nb)
        grad = wl.make_grad(cfg, tab, num_bags=nb)
        t0 = time.perf_counter()
        ora.forward(shape, cores, idx, off)
        ora.backward(shape, cores, idx, off, grad)
        return len(idx), time.perf_counter() - t0

    run(order[0], min(cfg.batch, 64))  # thread start-up and page faults stay out of the measurement
    probe_bags = min(cfg.batch, 2048)
    n, t = run(order[0], probe_bags)
    rate, mean_len = n / t, n / probe_bags   # lookups/s of the last run; lookups per bag
    total_n, total_t, used = 0, 0.0, []
    for tab in order:
        if total_t >= 10.0:
            break
        # whole batch if it fits into what is left of a ~25 s budget at the last measured rate
        fit = int(rate * (25.0 - total_t) / mean_len)
        nb = min(cfg.batch, max(64, fit))
        n, t = run(tab, nb)
        total_n += n
        total_t += t
        rate = n / t
        used.append("table %d: %s" % (tab, "whole batch" if nb == cfg.batch else "first %d bags" % nb))
    used = ["; ".join(used)]
    return {"value": total_n / total_t, "unit": "lookups/s", "cores": ora.max_threads(), "kind": "oracle",
            "sample": "definition-mode forward+backward, %s (%d lookups), %.1f s" % (used[0], total_n, total_t)}


if __name__ == "__main__":
    main()
