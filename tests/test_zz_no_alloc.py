"""The allocation-free forward entry point (reorder + planned forward in the library's static
device scratch) against the existing entry points it is a variant of: tt_index_reorder followed by
tt_emb_bag_forward with a caller workspace.  Two calls in a row on the shared scratch, the second
with a smaller input; bitwise equality, and the oracle's tolerance on top."""
import numpy as np
import pytest
import torch

import tt_workloads as wl

pytestmark = pytest.mark.gpu


def test_static_scratch_forward_equals_workspace_forward(ora):
    import gpu_util as g
    import paper_2507_14668_amd as tt
    from paper_2507_14668_amd import binding
    assert torch.cuda.is_available()
    cfg = wl.get_config(5)
    order = np.argsort([t.num_rows for t in cfg.tables])
    tab = int(order[len(order) // 2])
    shape, cores = cfg.tables[tab], wl.make_cores(cfg, tab)
    table = g.gpu_table(shape, cores)
    for call, nb in enumerate((20000, 3000)):  # the second call is smaller: stale scratch beyond it must not matter
        print("case static scratch call %d bags=%d" % (call, nb), flush=True)
        idx, off = wl.make_batch(cfg, tab, batch=call, num_bags=nb)
        d_idx, d_off = g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64)
        out = torch.full((nb, shape.dim), float("nan"), dtype=torch.float32, device="cuda")
        tt.tt_emb_bag_forward_static(table, d_idx, d_off, out)
        plan = tt.tt_index_reorder(table, d_idx, d_off)
        ref = tt.tt_emb_bag_forward(table, plan, d_idx, d_off)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "static-scratch forward differs from the workspace forward (call %d)" % call
        g.assert_close_rows(out.cpu().numpy(), ora.forward(shape, cores, idx, off, dedup=True), g.FWD_RTOL, shape.dim,
                            "static forward")
    # a batch beyond the static scratch is rejected, not truncated
    idx, off = wl.make_batch(cfg, tab, num_bags=65536)
    big = torch.empty((65536, shape.dim), dtype=torch.float32, device="cuda")
    with pytest.raises(tt.TTError) as e:
        tt.tt_emb_bag_forward_static(table, g.to_dev(idx, torch.int64), g.to_dev(off, torch.int64), big)
    assert e.value.status == binding.TT_ERR_WORKSPACE
