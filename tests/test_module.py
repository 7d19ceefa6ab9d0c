"""The nn.EmbeddingBag-style module: argument checks on the CPU, parity on the GPU (through the
same C ABI as everything else) against the direct calls, the oracle and a dense EmbeddingBag."""
import numpy as np
import pytest
import torch

import tt_workloads as wl


def test_module_argument_checks_and_shapes():
    import paper_2507_14668_amd as tt
    m = tt.TTEmbeddingBag(1000, 16, n=(10, 10, 10), d=(2, 2, 4), ranks=(4, 4), device="cpu")
    assert [p.numel() for p in m.parameters()] == [10 * 2 * 4, 4 * 10 * 2 * 4, 4 * 10 * 4]
    assert "smaller than dense" in repr(m)
    with pytest.raises(ValueError):
        tt.TTEmbeddingBag(1000, 16, n=(10, 10, 9), d=(2, 2, 4), ranks=(4, 4), device="cpu")
    with pytest.raises(ValueError):
        tt.TTEmbeddingBag(1000, 15, n=(10, 10, 10), d=(2, 2, 4), ranks=(4, 4), device="cpu")
    with pytest.raises(NotImplementedError):
        tt.TTEmbeddingBag(1000, 16, n=(10, 10, 10), d=(2, 2, 4), ranks=(4, 4), mode="mean", device="cpu")
    with pytest.raises(RuntimeError):  # no CPU path
        m(torch.zeros(4, dtype=torch.int64), torch.tensor([0, 2]))
    for rows in (1, 7, 1000, 1001, 12345, 40_000_000):
        n = tt.TTEmbeddingBag.near_cubic_factors(rows)
        assert n[0] * n[1] * n[2] >= rows and (n[0] - 1) * n[1] * n[2] < rows and max(n) - min(n) <= max(1, n[2])


def test_fused_collection_layout_on_cpu():
    """Construction only (no launch): families by (d, ranks), core values copied into the members' views."""
    import paper_2507_14668_amd as tt
    bags = [tt.TTEmbeddingBag(1000, 16, n=(10, 10, 10), d=(2, 2, 4), ranks=(4, 4), device="cpu"),
            tt.TTEmbeddingBag(60, 16, n=(3, 4, 5), d=(2, 2, 4), ranks=(3, 4), device="cpu"),
            tt.TTEmbeddingBag(60, 16, n=(3, 4, 5), d=(2, 2, 4), ranks=(4, 4), device="cpu")]
    coll = tt.TTEmbeddingBagCollection(bags, fuse=True)
    assert coll._where == [(0, 0), (1, 0), (0, 1)] and coll.fused[0].n == (13, 14, 15)
    for t, bag in enumerate(bags):
        gi, pos = coll._where[t]
        for k in range(3):
            assert torch.equal(coll.fused[gi].member_core(pos, k).contiguous().view(-1), bag.cores()[k])
    assert sum(p.numel() for p in coll.parameters()) == sum(p.numel() for b in bags for p in b.parameters())
    with pytest.raises(ValueError):
        tt.TTFusedEmbeddingBags([(10 ** 9, (1000, 1000, 1000)), (10 ** 9, (1000, 1000, 1000))], 16, (2, 2, 4), (4, 4), device="meta")


@pytest.fixture(scope="module")
def g():
    import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


def _module_like(tt, shape, cores, **kw):
    m = tt.TTEmbeddingBag(shape.num_rows, shape.dim, shape.n, shape.d, shape.r[1:3], **kw)
    with torch.no_grad():
        for p, c in zip(m.cores(), cores):
            p.copy_(torch.from_numpy(np.asarray(c, dtype=np.float32)))
    return m


@pytest.mark.gpu
@pytest.mark.parametrize("d,r", [((2, 3, 4), (1, 5, 6, 1)), ((4, 8, 4), (1, 32, 32, 1))])
def test_module_matches_direct_calls_and_oracle(g, ora, d, r):
    import paper_2507_14668_amd as tt
    print("case module d=%s r=%s" % (d, r), flush=True)
    shape, cores, idx, off, grad = wl.small_random_problem(91, n=(6, 5, 7), d=d, r=r, num_bags=400, max_len=6, sigma=0.2)
    d_idx, d_off, d_g = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), g.to_dev(grad, torch.float32)
    # direct calls
    table = g.gpu_table(shape, cores)
    plan = tt.tt_index_reorder(table, d_idx, d_off)
    out_ref = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
    dg_ref = tt.tt_emb_bag_backward(table, plan, d_idx, d_off, d_g)
    # module, offsets in both conventions
    for last in (True, False):
        m = _module_like(tt, shape, cores, include_last_offset=last)
        out = m(d_idx, d_off if last else d_off[:-1])
        assert torch.equal(out, out_ref)
        out.backward(d_g.view_as(out))
        for p, ref in zip(m.cores(), dg_ref):
            assert torch.equal(p.grad, ref)
    g.assert_close_rows(out.detach().cpu().numpy(), ora.forward(shape, cores, idx, off), g.FWD_RTOL, shape.dim, "module forward")
    g.assert_grads_close(shape, [p.grad for p in m.cores()], ora.backward(shape, cores, idx, off, grad), what="module dG")
    # an optimizer step on the module equals the oracle's update
    lr = 0.05
    torch.optim.SGD(m.parameters(), lr=lr).step()
    g.assert_grads_close(shape, [p.detach() for p in m.cores()], ora.sgd(cores, ora.backward(shape, cores, idx, off, grad), lr),
                         what="module SGD step")
    # fused mode: cores updated inside backward, bitwise equal to the fused direct call
    mf = _module_like(tt, shape, cores, include_last_offset=True, fused_sgd_lr=lr)
    of = mf(d_idx, d_off)
    of.backward(d_g.view_as(of))
    t2 = g.gpu_table(shape, cores)
    tt.tt_emb_bag_backward_sgd(t2, plan, d_idx, d_off, d_g, lr)
    torch.cuda.synchronize()
    for p, ref in zip(mf.cores(), t2.cores):
        assert p.grad is None and torch.equal(p.detach(), ref)


@pytest.mark.gpu
def test_module_two_dimensional_input_against_dense_embedding_bag(g):
    """2-D input (bags of equal length) and gradients of a downstream loss: the dense table the
    cores define, fed to torch.nn.functional.embedding_bag on the CPU in float64, must give the
    same outputs, and autograd through it the same core gradients."""
    import paper_2507_14668_amd as tt
    shape, cores, _, _, _ = wl.small_random_problem(92, n=(4, 3, 5), d=(2, 2, 2), r=(1, 3, 2, 1), num_bags=8, max_len=3, sigma=0.5)
    rng = np.random.default_rng(5)
    inp = rng.integers(0, shape.num_rows, size=(64, 5))
    m = _module_like(tt, shape, cores)
    out = m(torch.from_numpy(inp).cuda())
    w = torch.from_numpy(rng.standard_normal(out.shape).astype(np.float32)).cuda()
    (out * w).sum().backward()
    # dense route in float64
    c = [torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True) for x in cores]
    G1 = c[0].reshape(shape.n[0], shape.d[0], shape.r[1])
    G2 = c[1].reshape(shape.r[1], shape.n[1], shape.d[1], shape.r[2])
    G3 = c[2].reshape(shape.r[2], shape.n[2], shape.d[2])
    W = torch.einsum("iap,pjbq,qkc->ijkabc", G1, G2, G3).reshape(shape.n[0] * shape.n[1] * shape.n[2], shape.dim)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(inp), W, mode="sum")
    (ref * w.cpu().double()).sum().backward()
    g.assert_close_rows(out.detach().cpu().numpy(), ref.detach().numpy(), g.FWD_RTOL, shape.dim, "module 2-D forward")
    g.assert_grads_close(shape, [p.grad for p in m.cores()], [x.grad.reshape(-1).numpy() for x in c], what="module 2-D dG")


def test_collection_argument_checks():
    import paper_2507_14668_amd as tt
    kw = dict(num_embeddings=1000, embedding_dim=16, n=(10, 10, 10), d=(2, 2, 4), ranks=(4, 4), device="cpu")
    coll = tt.TTEmbeddingBagCollection([kw, tt.TTEmbeddingBag(**kw)], streams=2)
    assert len(coll.tables) == 2 and len(list(coll.parameters())) == 6
    with pytest.raises(ValueError):
        coll([torch.zeros(4, dtype=torch.int64)])  # one input per table
    with pytest.raises(ValueError):
        tt.TTEmbeddingBagCollection([kw], streams=0)


@pytest.mark.gpu
def test_collection_on_side_streams_equals_single_modules(g):
    """Three tables of different shapes dealt to two side streams: outputs and core gradients must
    equal, bit for bit, those of the same modules called one after the other on the current stream."""
    import paper_2507_14668_amd as tt
    problems = [wl.small_random_problem(400 + k, n=n, d=d, r=r, num_bags=300, max_len=4, sigma=0.3)
                for k, (n, d, r) in enumerate([((6, 5, 7), (2, 3, 4), (1, 5, 6, 1)),
                                               ((9, 3, 5), (4, 8, 4), (1, 32, 32, 1)),
                                               ((3, 4, 11), (4, 8, 4), (1, 64, 64, 1))])]
    results = []
    for streams in (1, 2):
        coll = tt.TTEmbeddingBagCollection([_module_like(tt, p[0], p[1]) for p in problems], streams=streams)
        inputs = [(torch.from_numpy(p[2]).cuda(), torch.from_numpy(p[3]).cuda()) for p in problems]
        for bag in coll.tables:
            bag.include_last_offset = True  # the generator's offsets are CSR (bags + 1 entries)
        outs = coll(inputs)
        loss = sum((o * torch.from_numpy(p[4]).cuda().view_as(o)).sum() for o, p in zip(outs, problems))
        loss.backward()
        torch.cuda.synchronize()
        results.append(([o.detach().clone() for o in outs], [p.grad.clone() for p in coll.parameters()]))
    for a, b in zip(results[0][0] + results[0][1], results[1][0] + results[1][1]):
        assert torch.equal(a, b)


@pytest.mark.gpu
def test_module_sample_route_and_bf16_inference(g, ora):
    """The module's other forward routes: sample-level reuse (same sums, gradients unchanged) and the
    bf16-core inference forward (against the oracle on cores rounded to bf16, fp32 tolerance)."""
    import paper_2507_14668_amd as tt
    from test_gpu_parity_small import round_to_bf16
    shape, cores, idx, off, grad = wl.small_random_problem(93, n=(6, 5, 7), d=(4, 8, 4), r=(1, 32, 32, 1), num_bags=500,
                                                          max_len=9, sigma=0.2)
    d_idx, d_off, d_g = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), g.to_dev(grad, torch.float32)
    ref_out = ora.forward(shape, cores, idx, off)
    ref_dg = ora.backward(shape, cores, idx, off, grad)
    m = _module_like(tt, shape, cores, include_last_offset=True, forward_route="sample")
    out = m(d_idx, d_off)
    g.assert_close_rows(out.detach().cpu().numpy(), ref_out, g.FWD_RTOL, shape.dim, "module forward (sample route)")
    out.backward(d_g.view_as(out))
    g.assert_grads_close(shape, [p.grad for p in m.cores()], ref_dg, what="module dG (sample route)")
    # bf16 inference: no graph, copies rebuilt on request
    out_b = m.forward_bf16(d_idx, d_off)
    assert not out_b.requires_grad
    rounded = [round_to_bf16(c) for c in cores]
    g.assert_close_rows(out_b.cpu().numpy(), ora.forward(shape, rounded, idx, off), g.FWD_RTOL, shape.dim,
                        "module forward_bf16")
    with torch.no_grad():
        m.core2.mul_(2.0)
    m.bf16_inference()
    doubled = [rounded[0], rounded[1], round_to_bf16(2.0 * np.asarray(cores[2], np.float32))]
    g.assert_close_rows(m.forward_bf16(d_idx, d_off).cpu().numpy(), ora.forward(shape, doubled, idx, off), g.FWD_RTOL,
                        shape.dim, "module forward_bf16 after refresh")
    with pytest.raises(ValueError):
        _module_like(tt, shape, cores, forward_route="nope")


@pytest.mark.gpu
@pytest.mark.parametrize("d,r", [((2, 3, 4), (1, 5, 6, 1)), ((4, 8, 4), (1, 32, 32, 1))])
def test_fused_module_matches_oracle_per_table(g, ora, d, r):
    """Several tables in one fused module: every table's outputs, autograd gradients and (fused-update
    mode) updated cores against the oracle on that table alone."""
    import paper_2507_14668_amd as tt
    print("case fused module d=%s r=%s" % (d, r), flush=True)
    ns = [(6, 5, 7), (3, 4, 2), (2, 9, 5)]
    probs = [wl.small_random_problem(200 + t, n=n, d=d, r=r, num_bags=60 + 25 * t, max_len=5, sigma=0.2) for t, n in enumerate(ns)]
    tables = [(p[0].num_rows, p[0].n) for p in probs]
    dim = d[0] * d[1] * d[2]

    def build(**kw):
        m = tt.TTFusedEmbeddingBags(tables, dim, d, r[1:3], **kw)
        with torch.no_grad():
            for t, p in enumerate(probs):
                for k in range(3):
                    m.member_core(t, k).copy_(torch.from_numpy(p[1][k]).view(p[0].core_shape(k)))
        return m

    inputs = [(g.to_dev(p[2], torch.int64), g.to_dev(p[3], torch.int64)[:-1]) for p in probs]
    m = build()
    outs = m(inputs)
    loss = sum((o * g.to_dev(p[4], torch.float32).view_as(o)).sum() for o, p in zip(outs, probs))
    loss.backward()
    for t, (shape, cores, idx, off, grad) in enumerate(probs):
        g.assert_close_rows(outs[t].detach().cpu().numpy(), ora.forward(shape, cores, idx, off), g.FWD_RTOL, shape.dim,
                            "fused module forward table %d" % t)
        got = [m.member_core(t, k, core=m.cores()[k].grad).contiguous().view(-1) for k in range(3)]
        g.assert_grads_close(shape, got, ora.backward(shape, cores, idx, off, grad), what="fused module dG table %d " % t)
    lr = 0.05
    mf = build(fused_sgd_lr=lr)
    outs_f = mf(inputs)
    sum((o * g.to_dev(p[4], torch.float32).view_as(o)).sum() for o, p in zip(outs_f, probs)).backward()
    torch.cuda.synchronize()
    assert all(c.grad is None for c in mf.cores())
    for t, (shape, cores, idx, off, grad) in enumerate(probs):
        got = [mf.member_core(t, k).detach().contiguous().view(-1) for k in range(3)]
        g.assert_grads_close(shape, got, ora.sgd(cores, ora.backward(shape, cores, idx, off, grad), lr),
                             what="fused module updated G table %d " % t)


@pytest.mark.gpu
def test_fused_collection_matches_oracle_per_table(g, ora):
    """A collection with `fuse=True`: tables of two families (different ranks) interleaved; each family
    becomes fused tables, outputs come back in table order and match the oracle table by table; the
    gradients of the fused cores, cut per table, match the oracle's."""
    import paper_2507_14668_amd as tt
    print("case fused collection", flush=True)
    specs = [((6, 5, 7), (4, 8, 4), (1, 32, 32, 1)), ((3, 4, 11), (2, 3, 4), (1, 5, 6, 1)), ((9, 3, 5), (4, 8, 4), (1, 32, 32, 1)),
             ((2, 2, 3), (2, 3, 4), (1, 5, 6, 1)), ((4, 4, 4), (4, 8, 4), (1, 32, 32, 1))]
    problems = [wl.small_random_problem(500 + k, n=n, d=d, r=r, num_bags=120 + 10 * k, max_len=4, sigma=0.3)
                for k, (n, d, r) in enumerate(specs)]
    coll = tt.TTEmbeddingBagCollection([_module_like(tt, p[0], p[1], include_last_offset=True) for p in problems],
                                       streams=2, fuse=True)
    assert len(coll.fused) == 2 and sorted(len(m.tables) for m in coll.fused) == [2, 3]
    inputs = [(torch.from_numpy(p[2]).cuda(), torch.from_numpy(p[3]).cuda()) for p in problems]
    outs = coll(inputs)
    loss = sum((o * torch.from_numpy(p[4]).cuda().view_as(o)).sum() for o, p in zip(outs, problems))
    loss.backward()
    torch.cuda.synchronize()
    for t, (shape, cores, idx, off, grad) in enumerate(problems):
        g.assert_close_rows(outs[t].detach().cpu().numpy(), ora.forward(shape, cores, idx, off), g.FWD_RTOL, shape.dim,
                            "fused collection forward table %d" % t)
        gi, pos = coll._where[t]
        m = coll.fused[gi]
        got = [m.member_core(pos, k, core=m.cores()[k].grad).contiguous().view(-1) for k in range(3)]
        g.assert_grads_close(shape, got, ora.backward(shape, cores, idx, off, grad), what="fused collection dG table %d " % t)
