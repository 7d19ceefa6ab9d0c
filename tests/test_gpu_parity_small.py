"""GPU parity (through the C ABI) against the CPU oracle: small shapes, configs 1-2, edge cases."""
import numpy as np
import pytest
import torch

import tt_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def run_all(g, ora, shape, cores, idx, off, grad, lr=0.01, check_plan=True, remap=None):
    import paper_2507_14668_amd as tt
    table = g.gpu_table(shape, cores)
    d_idx, d_off, d_grad = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), g.to_dev(grad, torch.float32)
    d_remap = None if remap is None else g.to_dev(remap, torch.int64)
    o_idx = idx if remap is None else np.where((idx >= 0) & (idx < shape.num_rows), remap[np.clip(idx, 0, shape.num_rows - 1)], -1)
    plan = tt.tt_index_reorder(table, d_idx, d_off, remap=d_remap)
    if check_plan:
        g.assert_plan_equals_oracle(ora, shape, plan, idx, off, remap=remap)
    ref_out = ora.forward(shape, cores, np.where(o_idx < 0, shape.num_rows, o_idx) if remap is not None else idx, off)
    out_plan = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    g.assert_close_rows(out_plan.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "forward(plan)")
    if remap is None:
        out_naive = tt.tt_emb_bag_forward(table, None, d_idx, d_off)
        g.assert_close_rows(out_naive.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "forward(naive)")
    # sample-level reuse route (Section III-B reuse equation): same bag sums, bitwise reproducible
    out_sample = tt.tt_emb_bag_forward_sample(table, plan, d_off)
    g.assert_close_rows(out_sample.cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "forward(sample)")
    assert torch.equal(tt.tt_emb_bag_forward_sample(table, plan, d_off), out_sample)
    ref_dg = ora.backward(shape, cores, np.where(o_idx < 0, shape.num_rows, o_idx) if remap is not None else idx, off, grad)
    dg_plan = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, d_grad)
    g.assert_grads_close(shape, dg_plan, ref_dg, what="dG(plan)")
    if remap is None:
        dg_naive = tt.tt_emb_bag_backward(table, None, d_idx, d_off, d_grad)
        g.assert_grads_close(shape, dg_naive, ref_dg, what="dG(naive)")
    # determinism of the planned arm: a second run is bitwise identical
    out2 = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    dg2 = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, d_grad)
    assert torch.equal(out2, out_plan)
    for k in range(3):
        assert torch.equal(dg2[k], dg_plan[k])
    # update: touched-slices arm and dense arm against the oracle
    ref_new = ora.sgd(cores, ref_dg, lr)
    t2 = g.gpu_table(shape, cores)
    tt.tt_core_sgd_update(table, plan, dg_plan, lr)
    tt.tt_core_sgd_update(t2, None, dg_plan, lr)
    torch.cuda.synchronize()
    for k in range(3):
        assert torch.equal(table.cores[k], t2.cores[k]), "touched-slice update differs from dense update"
    g.assert_grads_close(shape, table.cores, ref_new, what="updated G")
    # fused backward + update (Section III-F): bitwise the same cores as backward followed by update
    t3 = g.gpu_table(shape, cores)
    tt.tt_emb_bag_backward_sgd(t3, plan, d_idx, d_off, d_grad, lr)
    torch.cuda.synchronize()
    for k in range(3):
        assert torch.equal(t3.cores[k], table.cores[k]), "fused update differs from backward + update (core %d)" % k
    return plan


@pytest.mark.parametrize("seed,n,d,r,nb,ml", [
    (1, (3, 4, 5), (2, 3, 2), (1, 3, 4, 1), 40, 6),
    (2, (2, 2, 2), (2, 2, 2), (1, 2, 2, 1), 5, 3),
    (3, (5, 2, 7), (1, 4, 3), (1, 5, 2, 1), 300, 9),
    (4, (7, 6, 5), (4, 2, 4), (1, 8, 16, 1), 1000, 12),
    (5, (1, 1, 9), (2, 2, 2), (1, 1, 1, 1), 50, 4),
    (6, (2, 1, 1500), (2, 3, 2), (1, 3, 5, 1), 700, 4),   # a row factor above 1023: grouping sorts of two digits
    (7, (1, 3000, 3), (2, 3, 2), (1, 3, 4, 1), 900, 5),
    # capacity per i1 / i3 segment above 4096: the core-0 / core-2 reductions take the two-stage sum
    (8, (1, 5000, 2), (2, 3, 2), (1, 3, 5, 1), 4000, 7),
    (9, (1290, 1290, 1290), (2, 3, 2), (1, 3, 5, 1), 3000, 5),  # 31-bit row keys (2.1e9 rows): four radix passes
])
def test_small_shapes(g, ora, seed, n, d, r, nb, ml):
    print("case small_shapes seed=%d n=%s d=%s r=%s" % (seed, n, d, r), flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(seed, n=n, d=d, r=r, num_bags=nb, max_len=ml)
    run_all(g, ora, shape, cores, idx, off, grad)


@pytest.mark.parametrize("seed,n,r,nb,ml", [
    (61, (5, 7, 9), (1, 32, 32, 1), 300, 6),      # few prefixes per i2: partly filled chunks
    (62, (40, 3, 6), (1, 32, 32, 1), 2000, 8),    # > 16 prefixes per i2: several chunks
    (63, (3, 2, 50), (1, 64, 64, 1), 1500, 5),    # many rows per prefix, two column strips
    (64, (37, 5, 4), (1, 64, 64, 1), 900, 3),
    (66, (150, 2, 3), (1, 32, 32, 1), 1500, 3),   # > 64 prefixes per i2: staged plan entries are refilled
    (67, (150, 1, 5), (1, 64, 64, 1), 2500, 3),
    (68, (3, 2, 90), (1, 64, 64, 1), 1500, 5),    # up to 90 distinct rows per prefix: several row batches
    (69, (2, 3, 70), (1, 32, 32, 1), 1200, 4),
    (70, (1, 2100, 2), (1, 32, 32, 1), 1500, 3),  # a row factor above 1023: grouping sorts of two digits
    (71, (1, 2, 1100), (1, 64, 64, 1), 800, 4),
    # capacity per i1 / i3 segment above 4096: the core-0 / core-2 reductions take the two-stage sum
    (72, (1, 5000, 2), (1, 32, 32, 1), 4000, 7),
    (73, (2, 9000, 1), (1, 64, 64, 1), 5000, 5),
    (74, (1290, 1290, 1290), (1, 32, 32, 1), 3000, 5),  # 31-bit row keys (2.1e9 rows): four radix passes
])
def test_matrix_core_shapes(g, ora, seed, n, r, nb, ml):
    """Shapes served by the MFMA kernels (d = 4x8x4, ranks 32 or 64) on small tables."""
    print("case mfma shapes seed=%d n=%s r=%s" % (seed, n, r), flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(seed, n=n, d=(4, 8, 4), r=r, num_bags=nb,
                                                          max_len=ml, sigma=0.2)
    run_all(g, ora, shape, cores, idx, off, grad)


@pytest.mark.parametrize("rank,n2,split", [
    (64, 43, 2), (64, 42, 3), (64, 32, 4), (64, 25, 5), (64, 21, 6), (64, 18, 7), (64, 16, 8),
    (32, 100, 2), (32, 80, 3), (32, 64, 4), (32, 50, 5), (32, 42, 6), (32, 36, 7), (32, 32, 8),
])
def test_every_backward_split_factor(g, ora, rank, n2, split):
    """Tables with few core-1 slices deal the 8-prefix chunks of one (i2, strip) to 2..8 workgroups
    whose partial core-1 gradients a second kernel adds up: one case per factor and rank, with
    enough prefixes per i2 (up to 40) that parts get several chunks, one chunk, or none."""
    strips = 2 if rank == 64 else 1
    assert min(8, 256 // (n2 * strips)) == split and n2 * strips < 128
    print("case bwd split rank=%d n2=%d split=%d" % (rank, n2, split), flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(900 + rank + n2, n=(40, n2, 4), d=(4, 8, 4),
                                                          r=(1, rank, rank, 1), num_bags=2500, max_len=3, sigma=0.2)
    import paper_2507_14668_amd as tt
    table = g.gpu_table(shape, cores)
    d_idx, d_off, d_grad = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), g.to_dev(grad, torch.float32)
    plan = tt.tt_index_reorder(table, d_idx, d_off)
    g.assert_plan_equals_oracle(ora, shape, plan, idx, off)
    out = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    g.assert_close_rows(out.cpu().numpy(), ora.forward(shape, cores, idx, off, dedup=True), g.FWD_RTOL, shape.dim, "forward")
    dg = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, d_grad)
    ref_dg = ora.backward(shape, cores, idx, off, grad, dedup=True)
    g.assert_grads_close(shape, dg, ref_dg, what="dG")
    tt.tt_core_sgd_update(table, plan, dg, 0.01)
    fused = g.gpu_table(shape, cores)
    tt.tt_emb_bag_backward_sgd(fused, plan, d_idx, d_off, d_grad, 0.01)
    torch.cuda.synchronize()
    g.assert_grads_close(shape, fused.cores, ora.sgd(cores, ref_dg, 0.01), what="fused updated G")
    for k in range(3):
        assert torch.equal(fused.cores[k], table.cores[k]), "fused update differs from backward + update (core %d)" % k
    g.report_worst("split %d rank %d " % (split, rank))


def test_more_than_a_million_lookups(g, ora):
    """1.2 M lookups: the radix sort runs with more than 64 tiles (separate bin-scan launch) and the
    distinct-row pass with more than 1024 tiles (separate tile-sum scan launch).  Plan bit for bit,
    outputs and gradients against the dedup-mode oracle."""
    import paper_2507_14668_amd as tt
    print("case 1.2M lookups", flush=True)
    cfg = wl.get_config(1)
    shape, cores = cfg.tables[0], wl.make_cores(cfg, 0)
    rng = np.random.default_rng(77)
    nb = 300_000
    lens = rng.integers(0, 9, size=nb)
    off = np.zeros(nb + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    idx = rng.integers(0, shape.num_rows, size=int(off[-1]), dtype=np.int64)
    assert len(idx) > 1024 * 1024
    grad = rng.standard_normal(nb * shape.dim).astype(np.float32)
    table = g.gpu_table(shape, cores)
    d_idx, d_off = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64)
    plan = tt.tt_index_reorder(table, d_idx, d_off)
    g.assert_plan_equals_oracle(ora, shape, plan, idx, off)
    out = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    g.assert_close_rows(out.cpu().numpy(), ora.forward(shape, cores, idx, off, dedup=True), g.FWD_RTOL, shape.dim, "forward")
    dg = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, g.to_dev(grad, torch.float32))
    g.assert_grads_close(shape, dg, ora.backward(shape, cores, idx, off, grad, dedup=True), what="dG")
    g.report_worst("1.2M ")


def test_padded_table_and_remap(g, ora):
    print("case padded+remap", flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(11, n=(4, 5, 6), d=(2, 2, 4), r=(1, 4, 4, 1),
                                                          num_rows=101, num_bags=200, max_len=5)
    run_all(g, ora, shape, cores, idx, off, grad)
    remap = np.random.default_rng(2).permutation(shape.num_rows).astype(np.int64)
    run_all(g, ora, shape, cores, idx, off, grad, remap=remap)


@pytest.mark.parametrize("cfg_id", [1, 2])
def test_config_full(g, ora, cfg_id):
    print("case config %d" % cfg_id, flush=True)
    cfg = wl.get_config(cfg_id)
    shape, cores = cfg.tables[0], wl.make_cores(cfg, 0)
    idx, off = wl.make_batch(cfg, 0)
    run_all(g, ora, shape, cores, idx, off, wl.make_grad(cfg, 0), lr=cfg.lr)


def test_empty_batch_and_empty_bags(g, ora):
    print("case empty", flush=True)
    shape, cores, *_ = wl.small_random_problem(21)
    grad = np.random.default_rng(0).standard_normal(4 * shape.dim).astype(np.float32)
    run_all(g, ora, shape, cores, np.zeros(0, np.int64), np.zeros(5, np.int64), grad)
    run_all(g, ora, shape, cores, np.array([3, 3, 59], np.int64), np.array([0, 0, 2, 2, 3], np.int64), grad)


def test_hot_row_and_long_bag_span_many_chunks(g, ora):
    """One row repeated thousands of times (a segment spanning many reduction chunks) and one
    very long bag; also every lookup in one prefix."""
    print("case hot row", flush=True)
    shape, cores, *_ = wl.small_random_problem(22, n=(3, 4, 50), d=(2, 4, 4), r=(1, 8, 8, 1))
    rng = np.random.default_rng(1)
    idx = np.concatenate([np.full(5000, 7), rng.integers(0, 50, 3000), rng.integers(0, shape.num_rows, 500)]).astype(np.int64)
    rng.shuffle(idx)
    off = np.array([0, 6000, 6001, 8500], np.int64)
    off = np.concatenate([off[:-1], np.arange(6001, 8501, 1)[1:]]).astype(np.int64)
    nb = len(off) - 1
    grad = rng.standard_normal(nb * shape.dim).astype(np.float32)
    run_all(g, ora, shape, cores, idx, off, grad)


def test_invalid_indices_are_reported_and_skipped(g, ora):
    import paper_2507_14668_amd as tt
    from paper_2507_14668_amd import binding
    print("case invalid", flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(23, num_bags=60, max_len=5, num_rows=55)
    idx = idx.copy()
    idx[2], idx[17] = -3, 57  # 57 is inside the padded n1*n2*n3 range but >= num_rows
    plan = run_all(g, ora, shape, cores, idx, off, grad)
    assert tt.tt_plan_status(plan) == binding.TT_ERR_INDEX_RANGE
    table = g.gpu_table(shape, cores)
    good = np.abs(idx) % 55
    ok = tt.tt_index_reorder(table, g.to_dev(good, torch.int64), g.to_dev(off, torch.int64))
    assert tt.tt_plan_status(ok) == binding.TT_OK
    # offsets that are not monotone (still inside [0, nnz]) are reported; kernels clamp them
    bad_off = off.copy()
    k = int(np.argmax(np.diff(off) > 0))
    bad_off[k], bad_off[k + 1] = bad_off[k + 1], bad_off[k]
    bad = tt.tt_index_reorder(table, g.to_dev(good, torch.int64), g.to_dev(bad_off, torch.int64))
    counts, st = bad.counts()
    assert st == binding.TT_ERR_INDEX_RANGE and counts[3] & 2
    out = tt.tt_emb_bag_forward(table, bad, g.to_dev(good, torch.int64), g.to_dev(bad_off, torch.int64))
    assert torch.isfinite(out).all()
    out = tt.tt_emb_bag_forward_sample(table, bad, g.to_dev(bad_off, torch.int64))
    assert torch.isfinite(out).all()


def test_host_side_argument_errors(g):
    import paper_2507_14668_amd as tt
    from paper_2507_14668_amd import binding
    shape, cores, idx, off, grad = wl.small_random_problem(24)
    table = g.gpu_table(shape, cores)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(tt.TTError) as e:
        tt.tt_index_reorder(table, g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), workspace=small)
    assert e.value.status == binding.TT_ERR_WORKSPACE
    bad = tt.Table(shape.num_rows, shape.n, shape.d, shape.r, table.cores)
    bad.c.r[0] = 2
    with pytest.raises(tt.TTError) as e:
        tt.tt_emb_bag_forward(bad, None, g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64))
    assert e.value.status == binding.TT_ERR_SHAPE
    # the fused backward + update needs a plan (the naive arm has no point where a slice is complete)
    with pytest.raises(tt.TTError) as e:
        tt.tt_emb_bag_backward_sgd(table, None, g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64),
                                   g.to_dev(grad, torch.float32), 0.01)
    assert e.value.status == binding.TT_ERR_INVALID_ARG


def test_unaligned_core_and_gradient_buffers_take_the_scalar_paths(g, ora):
    """Cores and gradient buffers that are only 4-byte aligned (views into larger tensors) must
    give the same results: the matrix-core kernels and the float4 stores are then bypassed."""
    import paper_2507_14668_amd as tt
    print("case unaligned", flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(65, n=(6, 4, 5), d=(4, 8, 4), r=(1, 32, 32, 1), num_bags=200,
                                                          max_len=5, sigma=0.2)
    d_idx, d_off, d_g = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), g.to_dev(grad, torch.float32)
    views = []
    for c in cores:  # every core starts one float past a 16-byte boundary
        buf = torch.empty(len(c) + 1, dtype=torch.float32, device="cuda")
        buf[1:].copy_(torch.from_numpy(np.asarray(c, dtype=np.float32)))
        views.append(buf[1:])
    table = tt.Table(shape.num_rows, shape.n, shape.d, shape.r, views)
    plan = tt.tt_index_reorder(table, d_idx, d_off)
    out = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    g.assert_close_rows(out.cpu().numpy(), ora.forward(shape, cores, idx, off), g.FWD_RTOL, shape.dim, "unaligned forward")
    dviews = [torch.empty(len(c) + 1, dtype=torch.float32, device="cuda")[1:] for c in cores]
    tt.tt_emb_bag_backward(table, plan, d_idx, d_off, d_g, dcores=dviews)
    ref_dg = ora.backward(shape, cores, idx, off, grad)
    g.assert_grads_close(shape, dviews, ref_dg, what="unaligned dG")
    # the fused backward + update writes into the (unaligned) cores themselves
    tt.tt_core_sgd_update(table, plan, dviews, 0.01)
    fviews = []
    for c in cores:
        buf = torch.empty(len(c) + 1, dtype=torch.float32, device="cuda")
        buf[1:].copy_(torch.from_numpy(np.asarray(c, dtype=np.float32)))
        fviews.append(buf[1:])
    ftable = tt.Table(shape.num_rows, shape.n, shape.d, shape.r, fviews)
    tt.tt_emb_bag_backward_sgd(ftable, plan, d_idx, d_off, d_g, 0.01)
    torch.cuda.synchronize()
    for k in range(3):
        assert torch.equal(fviews[k], views[k]), "unaligned fused update differs from backward + update (core %d)" % k
    g.assert_grads_close(shape, fviews, ora.sgd(cores, ref_dg, 0.01), what="unaligned fused updated G")
    # aligned cores (matrix-core kernels, split workgroups) with an unaligned core-1 gradient buffer
    table2 = g.gpu_table(shape, cores)
    plan2 = tt.tt_index_reorder(table2, d_idx, d_off)
    mixed = table2.core_grads_like()
    mixed[1] = torch.empty(len(cores[1]) + 1, dtype=torch.float32, device="cuda")[1:]
    tt.tt_emb_bag_backward(table2, plan2, d_idx, d_off, d_g, dcores=mixed)
    g.assert_grads_close(shape, mixed, ref_dg, what="unaligned dG2 buffer")


def round_to_bf16(a):
    """fp32 -> nearest bf16 (ties to even), returned as fp32: the storage format of the reduced-precision
    cores, written here from the format's definition (upper 16 bits of the fp32 pattern)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def check_bf16_forward(g, ora, shape, cores, idx, off, what):
    import paper_2507_14668_amd as tt
    table = g.gpu_table(shape, cores)
    d_idx, d_off = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64)
    plan = tt.tt_index_reorder(table, d_idx, d_off)
    bf = tt.tt_cores_to_bf16(table)
    out = tt.tt_emb_bag_forward_bf16(table, bf, plan, d_off).cpu().numpy()
    rounded = [round_to_bf16(c) for c in cores]
    # (1) fp32 accumulation of exactly representable products: the oracle on the rounded cores, fp32 tolerance
    ref_rounded = ora.forward(shape, rounded, idx, off, dedup=True)
    g.assert_close_rows(out, ref_rounded, g.FWD_RTOL, shape.dim, "%s bf16 forward vs oracle(rounded cores)" % what)
    # (2) against the unrounded cores: every core element moves by at most 2^-9 relative, so every
    # TT path product by at most (1 + 2^-9)^3 - 1, and the bag sum by that times the sum of |paths|
    # = the oracle's forward of the absolute cores
    ref = ora.forward(shape, cores, idx, off, dedup=True).astype(np.float64)
    path_sum = ora.forward(shape, [np.abs(c) for c in cores], idx, off, dedup=True).astype(np.float64)
    bound = ((1 + 2.0 ** -9) ** 3 - 1) * path_sum + g.FWD_RTOL * np.abs(ref).max()
    assert np.all(np.abs(out - ref) <= bound), "%s: bf16 storage error above its bound" % what
    rel = np.abs(out - ref).max() / np.abs(ref).max()
    print("  %s: bf16-core forward differs from the fp32-core oracle by %.2e of the largest output" % (what, rel), flush=True)
    assert rel > 1e-5, "the rounding of the cores must be visible (is the bf16 path really bf16?)"
    # unsupported shapes are refused, not silently served in fp32
    return plan


@pytest.mark.parametrize("seed,n,r,nb,ml", [
    (71, (5, 7, 9), (1, 32, 32, 1), 300, 6),
    (72, (150, 2, 3), (1, 32, 32, 1), 1500, 3),
    (73, (3, 2, 90), (1, 64, 64, 1), 1500, 5),
    (74, (37, 5, 4), (1, 64, 64, 1), 900, 3),
])
def test_bf16_cores_forward(g, ora, seed, n, r, nb, ml):
    """Reduced-precision storage of the cores (bf16) with fp32 accumulation, on the matrix-core shapes."""
    print("case bf16 seed=%d n=%s r=%s" % (seed, n, r), flush=True)
    shape, cores, idx, off, _ = wl.small_random_problem(seed, n=n, d=(4, 8, 4), r=r, num_bags=nb, max_len=ml, sigma=0.2)
    check_bf16_forward(g, ora, shape, cores, idx, off, "small")


@pytest.mark.parametrize("cfg_id,tab", [(3, 0), (5, 1)])
def test_bf16_cores_forward_config_tables(g, ora, cfg_id, tab):
    print("case bf16 cfg%d table %d" % (cfg_id, tab), flush=True)
    cfg = wl.get_config(cfg_id)
    shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
    idx, off = wl.make_batch(cfg, tab)
    check_bf16_forward(g, ora, shape, cores, idx, off, "cfg%d" % cfg_id)


def test_bf16_cores_refused_for_other_shapes(g):
    import paper_2507_14668_amd as tt
    shape, cores, *_ = wl.small_random_problem(75)
    table = g.gpu_table(shape, cores)
    assert tt.tt_bf16_cores_bytes(table) == 0
    with pytest.raises(tt.TTError):
        tt.tt_cores_to_bf16(table)


def test_seeded_random_shapes(g, ora):
    """Sixty seeded random shapes and batches within the library's limits (ranks and factors that are not
    powers of two, single-slice cores, padded row counts, the matrix-core shapes, bags of up to 70
    lookups, batches of up to 3000 bags): every entry point of the planned and naive arms against the
    oracle, the plan bit for bit, the fused update bit for bit against backward + update."""
    rng = np.random.default_rng(20250715)
    for case in range(60):
        while True:
            n = tuple(int(x) for x in rng.integers(1, 40, size=3))
            d = tuple(int(x) for x in rng.choice([1, 2, 3, 4, 5, 8], size=3))
            r1, r2 = int(rng.choice([1, 2, 3, 7, 16, 33, 64])), int(rng.choice([1, 2, 5, 8, 17, 32, 64]))
            if rng.random() < 0.3:
                d, r1 = (4, 8, 4), int(rng.choice([32, 64]))
                r2 = r1
            dim, p12, s2 = d[0] * d[1] * d[2], d[0] * d[1] * r2, d[1] * r2
            lds = d[0] * r1 + d[0] * d[1] * (r2 | 1) + p12 + dim + 8 * r2 * d[2]
            if dim <= 1024 and p12 <= 4096 and s2 <= 4096 and lds * 4 <= 65536:
                break
        cap = n[0] * n[1] * n[2]
        num_rows = int(rng.integers(max(1, cap - n[2] + 1), cap + 1))
        nb = int(rng.choice([1, 7, 100, 700, 3000]))
        ml = int(rng.choice([1, 3, 9, 70]))
        if nb * ml > 40000:
            nb = 40000 // ml
        print("case random %d n=%s d=%s r=(%d,%d) rows=%d bags=%d max_len=%d" % (case, n, d, r1, r2, num_rows, nb, ml), flush=True)
        shape, cores, idx, off, grad = wl.small_random_problem(8000 + case, n=n, d=d, r=(1, r1, r2, 1), num_rows=num_rows,
                                                              num_bags=nb, max_len=ml, sigma=0.3)
        if case % 3 == 0 and len(idx):  # skew: a third of the cases look mostly at a few rows
            hot = rng.integers(0, num_rows, size=3)
            mask = rng.random(len(idx)) < 0.7
            idx = np.where(mask, hot[rng.integers(0, 3, len(idx))], idx).astype(np.int64)
        run_all(g, ora, shape, cores, idx, off, grad)
