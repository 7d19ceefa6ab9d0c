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


def _header_struct_fields(name):
    """(field, array suffix) of every member of `typedef struct { ... } name;` in the header."""
    text = open(os.path.join(ROOT, "include", "tt_emb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    body = re.search(r"typedef struct \{([^}]*)\} %s;" % name, text).group(1)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        for part in decl.split(","):
            m = re.search(r"(\w+)\s*((?:\[\w+\])*)\s*$", part.strip())
            fields.append((m.group(1), m.group(2)))
    return fields


def test_struct_mirrors_match_header_layout(tmp_path):
    """The ctypes mirrors of the public structs are pinned to the header: a C program that includes
    include/tt_emb.h prints sizeof and offsetof of every member (names parsed from the header), and
    the ctypes classes must have the same members at the same offsets."""
    import subprocess
    from paper_2507_14668_amd import binding
    pairs = (("tt_table", binding.CTable), ("tt_plan", binding.CPlan), ("tt_batch_item", binding.CBatchItem),
             ("tt_fuse_members", binding.CFuseMembers))
    lines = ["#include <stdio.h>", "#include <stddef.h>", '#include "tt_emb.h"', "int main(void) {"]
    for cname, _ in pairs:
        lines.append('printf("%s sizeof %%zu\\n", sizeof(%s));' % (cname, cname))
        for field, _n in _header_struct_fields(cname):
            lines.append('printf("%s %s %%zu\\n", offsetof(%s, %s));' % (cname, field, cname, field))
    lines.append("return 0; }")
    src, exe = tmp_path / "layout.c", tmp_path / "layout"
    src.write_text("\n".join(lines))
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = {}
    for ln in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines():
        cname, field, off = ln.split()
        got[(cname, field)] = int(off)
    for cname, cls in pairs:
        assert ctypes.sizeof(cls) == got[(cname, "sizeof")], cname
        header_fields = [f for f, _ in _header_struct_fields(cname)]
        assert [f for f, _ in cls._fields_] == header_fields, cname
        for field in header_fields:
            assert getattr(cls, field).offset == got[(cname, field)], (cname, field)


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


def test_fused_table_shape_and_host_validation_without_gpu():
    """tt_fuse_shape is host arithmetic; tt_fuse_lookups rejects bad arguments before any launch."""
    from paper_2507_14668_amd import binding
    lib = binding.load_library()
    assert binding.TT_FUSE_MAX_TABLES == int(re.search(r"#define TT_FUSE_MAX_TABLES (\d+)",
                                                       open(os.path.join(ROOT, "include", "tt_emb.h")).read()).group(1))
    layout = binding.FusedLayout([(1000, (10, 10, 10)), (55, (3, 4, 5)), (8, (2, 2, 2))])
    assert layout.n == (15, 16, 17) and layout.num_rows == 15 * 16 * 17
    assert layout.start == [[0, 0, 0], [10, 10, 10], [13, 14, 15]]
    assert layout.bag_ranges([4, 0, 7]) == [(0, 4), (4, 4), (4, 11)]
    m = binding.CFuseMembers()
    t = binding.CTable()
    assert lib.tt_fuse_shape(ctypes.byref(m), ctypes.byref(t)) == binding.TT_ERR_INVALID_ARG  # no members
    m.num_tables = 2
    for k in range(2):
        m.n[k][:] = (1200, 1200, 1200)
        m.num_rows[k] = 1200 ** 3
    assert lib.tt_fuse_shape(ctypes.byref(m), ctypes.byref(t)) == binding.TT_ERR_SHAPE  # 2400^3 rows
    m.n[1][:] = (3, 4, 5)
    m.num_rows[1] = 61
    assert lib.tt_fuse_shape(ctypes.byref(m), ctypes.byref(t)) == binding.TT_ERR_SHAPE  # more rows than 3*4*5
    m.num_rows[1] = 60
    assert lib.tt_fuse_shape(ctypes.byref(m), ctypes.byref(t)) == 0 and tuple(t.n) == (1203, 1204, 1205)
    assert lib.tt_fuse_lookups(ctypes.byref(m), None, None, None, None, None, None, None, None) == binding.TT_ERR_INVALID_ARG
    # deal-out helper: largest first, balanced, within the limits
    members = [(n ** 3, (n, n, n)) for n in (10, 342, 26, 44, 500, 900, 31)]
    parts = binding.fusion_groups(members)
    assert sorted(t for p in parts for t in p) == list(range(7))
    for p in parts:
        assert sum(members[t][1][0] for t in p) <= 1023
    assert len(binding.fusion_groups(members, groups=5)) == 5
