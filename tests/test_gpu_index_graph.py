"""GPU parity of the index-graph edge job (Section III-G, index-graph generation) through the C ABI:
bit-exact against the loop oracle on small batches, against the host construction at config-3 size,
and the reuse the bijection built from GPU edges buys (the only yardstick the paper leaves)."""
import numpy as np
import pytest
import torch

import tt_workloads as wl

pytestmark = pytest.mark.gpu


def gpu_edges(idx, off, rank, hot, max_group, max_pairs=None):
    import paper_2507_14668_amd as tt
    u, v, w = tt.tt_index_graph_edges(torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda(),
                                      torch.from_numpy(np.ascontiguousarray(rank, dtype=np.int32)).cuda(), hot, max_group,
                                      max_pairs=max_pairs)
    return u.cpu().numpy(), v.cpu().numpy(), w.cpu().numpy()


@pytest.mark.parametrize("nb,ml,rows,hot,max_group", [
    (300, 9, 400, 5, 64),        # short bags
    (2000, 40, 100000, 50, 64),  # several sort tiles, 17-bit keys
    (40, 300, 3000, 0, 16),      # bags longer than a wavefront round and than the 256-lookup cap; group limit
    (200, 5, 50, 45, 64),        # almost every row hot
    (5, 0, 10, 0, 64),           # no lookup at all
])
def test_edges_equal_loop_oracle(ora, nb, ml, rows, hot, max_group):
    print("case index graph nb=%d ml=%d rows=%d hot=%d max_group=%d" % (nb, ml, rows, hot, max_group), flush=True)
    rng = np.random.default_rng(nb + ml)
    lens = rng.integers(0, ml + 1, nb)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.minimum((rows ** rng.random(int(off[-1]))).astype(np.int64), rows - 1)
    idx[::17] = -1  # invalid lookups are skipped
    rank = rng.permutation(rows).astype(np.int32)
    ref = ora.index_graph_edges(idx, off, rank, hot, max_group)
    u, v, w = gpu_edges(idx, off, rank, hot, max_group)
    got = {(int(a), int(b)): int(c) for a, b, c in zip(u, v, w)}
    assert got == ref
    keys = list(zip(u.tolist(), v.tolist()))
    assert keys == sorted(keys) and len(set(keys)) == len(keys)
    if sum(ref.values()) > 1:  # a capacity below the pair count is reported
        import paper_2507_14668_amd as tt
        with pytest.raises(tt.TTError):
            gpu_edges(idx, off, rank, hot, max_group, max_pairs=sum(ref.values()) - 1)


def test_edges_of_a_config3_batch_equal_host_construction():
    """One table of config 3 at its full batch (16384 multi-hot bags, 3.2 million pairs): the GPU edge
    list against the numpy construction of the package (itself compared with the loop oracle below on
    a prefix of the bags), bit for bit."""
    from oracle import tt_oracle as ora
    from paper_2507_14668_amd import bijection as bj
    cfg = wl.get_config(3)
    shape = cfg.tables[0]
    idx, off = wl.make_batch(cfg, 0, permute_rows=True)
    rank, _ = bj.frequency_order([idx], shape.num_rows)
    hot = 100
    print("case index graph cfg3 nnz=%d" % len(idx), flush=True)
    u, v, w = gpu_edges(idx, off, rank, hot, 64)
    hu, hv, hw = bj.index_graph_edges([(idx, off)], rank, hot)
    assert np.array_equal(u, hu) and np.array_equal(v, hv) and np.array_equal(w, hw)
    nb = 300
    ref = ora.index_graph_edges(idx[:off[nb]], off[:nb + 1], rank, hot, 64)
    pu, pv, pw = gpu_edges(idx[:off[nb]].copy(), off[:nb + 1].copy(), rank, hot, 64)
    assert {(int(a), int(b)): int(c) for a, b, c in zip(pu, pv, pw)} == ref
    print("  %d edges from %d pairs" % (len(u), int(w.sum())), flush=True)


def test_bijection_from_gpu_edges_lowers_distinct_prefixes():
    """Planted communities scattered over the index space: the bijection built from GPU-generated edges
    is the same permutation as the one from host edges and gives fewer distinct prefixes per held-out batch."""
    from paper_2507_14668_amd import bijection as bj
    from test_bijection import _planted
    num_rows, n = 120000, (60, 100, 20)
    batches = _planted(2, num_rows=num_rows, ncomm=2400, nbatch=66)
    train, held_out = batches[:60], batches[60:]
    remap_gpu = bj.build_index_bijection(train, num_rows, hot_ratio=0.0002, seed=0, device="cuda")
    remap_cpu = bj.build_index_bijection(train, num_rows, hot_ratio=0.0002, seed=0)
    assert np.array_equal(remap_gpu, remap_cpu)
    _, pref0 = bj.prefix_reuse_stats(held_out, n)
    _, pref1 = bj.prefix_reuse_stats(held_out, n, remap_gpu)
    print("  distinct prefixes per batch: %.0f -> %.0f" % (pref0, pref1), flush=True)
    assert pref1 < 0.7 * pref0
