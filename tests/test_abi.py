"""The C-ABI library loads and exports every symbol include/tt_emb.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tt_emb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tt_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = declared_functions()
    for must in ("tt_index_reorder", "tt_emb_bag_forward", "tt_emb_bag_backward", "tt_core_sgd_update"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2507_14668_amd import binding
    lib = binding.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(declared_functions())
    assert binding.strerror(0) == "ok" and "workspace" in binding.strerror(binding.TT_ERR_WORKSPACE)


def test_struct_mirrors_match_header_sizes():
    from paper_2507_14668_amd import binding
    # tt_table: int64 + 3*int32 + 3*int32 + 4*int32 + 3 pointers = 8 + 40 + 24 = 72 bytes
    assert ctypes.sizeof(binding.CTable) == 72
    # tt_plan: 4*int64 + 10*int32 (+pad) + 18 + 7 + 3 pointers + size_t
    assert ctypes.sizeof(binding.CPlan) == 32 + 40 + 8 * (20 + 8 + 3) + 8


def test_workspace_query_and_host_validation_without_gpu():
    from paper_2507_14668_amd import binding
    lib = binding.load_library()
    t = binding.CTable()
    t.num_rows = 1000
    t.n[:] = (10, 10, 10)
    t.d[:] = (2, 2, 4)
    t.r[:] = (1, 4, 4, 1)
    small = lib.tt_workspace_bytes(ctypes.byref(t), 256, 256)
    big = lib.tt_workspace_bytes(ctypes.byref(t), 4096, 256)
    assert 0 < small < big and small % 256 == 0
    assert lib.tt_workspace_bytes(ctypes.byref(t), -1, 256) == 0
    t.r[0] = 2
    assert lib.tt_workspace_bytes(ctypes.byref(t), 256, 256) == 0
    # argument errors are detected on the host before anything touches a device
    t.r[0] = 1
    plan = binding.CPlan()
    st = lib.tt_index_reorder(ctypes.byref(t), None, None, 4, 4, None, None, 0, ctypes.byref(plan), None)
    assert st == binding.TT_ERR_INVALID_ARG
    st = lib.tt_emb_bag_forward(None, None, None, None, 0, 0, None, None)
    assert st == binding.TT_ERR_INVALID_ARG


def test_batched_entry_points_are_switched_off():
    """They report TT_ERR_UNAVAILABLE and launch nothing (see the header for the reason)."""
    from paper_2507_14668_amd import binding
    lib = binding.load_library()
    items = (binding.CBatchItem * 1)()
    for name in ("tt_index_reorder_batched", "tt_emb_bag_forward_batched", "tt_emb_bag_backward_batched"):
        assert getattr(lib, name)(1, items, None, 0, None) == binding.TT_ERR_UNAVAILABLE
    assert lib.tt_core_sgd_update_batched(1, items, 0.1, None, 0, None) == binding.TT_ERR_UNAVAILABLE
    assert lib.tt_batch_desc_bytes(4) > 0
