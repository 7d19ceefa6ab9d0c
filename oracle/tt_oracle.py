"""ctypes front-end of the CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT PATH.

Only `tests/`, `__graft_entry__.smoke()` and `bench.py`'s `cpu_baseline` leg may
import this module.  It loads `libtt_oracle.so` (plain C, built from
`tt_oracle.c` by `build_oracle()`), and adds the integer reorder-plan oracle,
which is the plain definition written with library sort / unique routines.

Nothing here imports, calls or shares code with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tt_oracle.c")
_LIB = os.path.join(_HERE, "libtt_oracle.so")
_lib = None


class _OraTable(ctypes.Structure):
    _fields_ = [("num_rows", ctypes.c_int64), ("n", ctypes.c_int32 * 3), ("d", ctypes.c_int32 * 3),
                ("r", ctypes.c_int32 * 4), ("g1", ctypes.c_void_p), ("g2", ctypes.c_void_p),
                ("g3", ctypes.c_void_p)]


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (building the checker is not using it)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        lib.ora_max_threads.restype = ctypes.c_int
        lib.ora_split_index.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.ora_row.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        for name in ("ora_forward", "ora_forward_dedup"):
            f = getattr(lib, name)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                          ctypes.c_int64, ctypes.c_void_p]
        for name in ("ora_backward", "ora_backward_dedup"):
            f = getattr(lib, name)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                          ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                          ctypes.c_void_p, ctypes.c_void_p]
        lib.ora_sgd.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_float]
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().ora_max_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32).reshape(-1)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64).reshape(-1)


def _table(shape, cores):
    g = [_f32(c) for c in cores]
    for k in range(3):
        assert g[k].size == shape.r[k] * shape.n[k] * shape.d[k] * shape.r[k + 1], "core %d size" % k
    assert shape.r[0] == 1 and shape.r[3] == 1
    t = _OraTable()
    t.num_rows = int(shape.num_rows)
    t.n[:] = list(shape.n)
    t.d[:] = list(shape.d)
    t.r[:] = list(shape.r)
    t.g1, t.g2, t.g3 = (x.ctypes.data for x in g)
    return t, g  # keep g alive while t is in use


def split_index(idx: int, n) -> tuple:
    nn = (ctypes.c_int32 * 3)(*n)
    out = (ctypes.c_int64 * 3)()
    _load().ora_split_index(int(idx), nn, out)
    return tuple(int(x) for x in out)


def row(shape, cores, idx: int) -> np.ndarray:
    """One reconstructed embedding row, float64[D]."""
    t, keep = _table(shape, cores)
    out = np.zeros(shape.dim, dtype=np.float64)
    _load().ora_row(ctypes.byref(t), int(idx), out.ctypes.data)
    return out


def forward(shape, cores, indices, offsets, dedup: bool = False) -> np.ndarray:
    """Bag sums, float32[B][D].  `dedup` selects the re-associated (fast) mode."""
    t, keep = _table(shape, cores)
    idx, off = _i64(indices), _i64(offsets)
    nb = off.size - 1
    assert off[0] == 0 and off[-1] == idx.size and np.all(np.diff(off) >= 0)
    out = np.zeros((nb, shape.dim), dtype=np.float32)
    f = _load().ora_forward_dedup if dedup else _load().ora_forward
    f(ctypes.byref(t), idx.ctypes.data, off.ctypes.data, idx.size, nb, out.ctypes.data)
    return out


def backward(shape, cores, indices, offsets, grad_out, dedup: bool = False, max_threads_: int = 0):
    """TT-core gradients [dG1, dG2, dG3] (flat float32, core-shaped)."""
    t, keep = _table(shape, cores)
    idx, off, g = _i64(indices), _i64(offsets), _f32(grad_out)
    nb = off.size - 1
    assert g.size == nb * shape.dim
    assert off[0] == 0 and off[-1] == idx.size and np.all(np.diff(off) >= 0)
    dg = [np.zeros(keep[k].size, dtype=np.float32) for k in range(3)]
    f = _load().ora_backward_dedup if dedup else _load().ora_backward
    rc = f(ctypes.byref(t), idx.ctypes.data, off.ctypes.data, idx.size, nb, g.ctypes.data,
           int(max_threads_), dg[0].ctypes.data, dg[1].ctypes.data, dg[2].ctypes.data)
    if rc < 0:
        raise MemoryError("oracle backward: accumulator allocation failed")
    return dg


def sgd(cores, dcores, lr: float):
    """Plain gradient descent, returns new cores (inputs untouched)."""
    out = []
    for g, dg in zip(cores, dcores):
        gg = _f32(g).copy()
        d = _f32(dg)
        _load().ora_sgd(gg.ctypes.data, d.ctypes.data, gg.size, ctypes.c_float(lr))
        out.append(gg)
    return out


def reorder_plan(shape, indices, offsets, remap=None) -> dict:
    """Integer oracle of the index-reordering pass (Sections III-C, III-E, III-G).

    The lookups are (optionally remapped by the index bijection, then) stably
    sorted by row; ties keep their original position, so the plan is unique.
    Distinct rows and distinct (i1,i2) prefixes (prefix = row div n3, the key
    of the paper's reuse buffer) are listed in increasing order.  Invalid
    indices (negative or >= num_rows) take no part in the plan.
    """
    idx = _i64(indices)
    off = _i64(offsets)
    nnz = idx.size
    rows = idx if remap is None else np.where((idx >= 0) & (idx < len(remap)),
                                              _i64(remap)[np.clip(idx, 0, len(remap) - 1)], -1)
    valid = (rows >= 0) & (rows < shape.num_rows)
    bag_of_lookup = np.repeat(np.arange(off.size - 1, dtype=np.int64), np.diff(off))
    pos = np.nonzero(valid)[0]
    order = pos[np.argsort(rows[pos], kind="stable")]
    sorted_row = rows[order]
    uniq_row, first, inverse = np.unique(sorted_row, return_index=True, return_inverse=True)
    row_seg = np.concatenate([first, [sorted_row.size]]).astype(np.int64)
    lookup2row = np.full(nnz, -1, dtype=np.int64)
    lookup2row[order] = inverse
    pref_of_row = uniq_row // shape.n[2]
    uniq_pref, pfirst, row2pref = np.unique(pref_of_row, return_index=True, return_inverse=True)
    pref_seg = np.concatenate([pfirst, [uniq_row.size]]).astype(np.int64)
    return dict(perm=order, sorted_row=sorted_row, bag_of_sorted=bag_of_lookup[order],
                uniq_row=uniq_row, row_seg=row_seg, lookup2row=lookup2row,
                uniq_pref=uniq_pref, pref_seg=pref_seg, row2pref=row2pref,
                num_valid=int(sorted_row.size), any_invalid=bool((~valid).any()))


def forward_sample_reuse(shape, cores, indices, offsets):
    """Bag sums by the sample-level reuse equation of Section III-B, float64[B][D], and the number
    of (bag, prefix) groups it formed.

    Inside one bag, the lookups whose rows share the first two TT indices (i1, i2) are served
    by ONE product chain: the shared slices G1[i1] and G2[i2] are multiplied once, and the
    third factor is the SUM of the core-3 slices of those lookups,
        sum_l G1[i1] G2[i2] G3[i3_l]  =  G1[i1] G2[i2] (sum_l G3[i3_l]).
    It is the same bag sum as `forward` in another association order; everything is float64
    here, so the two agree to rounding.  Invalid indices contribute nothing.
    """
    n1, n2, n3 = shape.n
    d1, d2, d3 = shape.d
    _, r1, r2, _ = shape.r
    g1 = np.asarray(cores[0], dtype=np.float64).reshape(n1, d1, r1)
    g2 = np.asarray(cores[1], dtype=np.float64).reshape(r1, n2, d2, r2)
    g3 = np.asarray(cores[2], dtype=np.float64).reshape(r2, n3, d3)
    idx, off = _i64(indices), _i64(offsets)
    nb = off.size - 1
    out = np.zeros((nb, d1 * d2 * d3), dtype=np.float64)
    groups = 0
    for b in range(nb):
        slice_sum = {}  # (i1, i2) -> sum of the core-3 slices of the bag's lookups with that prefix
        for i in idx[off[b]:off[b + 1]]:
            if i < 0 or i >= shape.num_rows:
                continue
            i3 = int(i % n3)
            i2 = int((i // n3) % n2)
            i1 = int(i // (n2 * n3))
            s = slice_sum.get((i1, i2))
            slice_sum[(i1, i2)] = g3[:, i3, :].copy() if s is None else s + g3[:, i3, :]
        for (i1, i2), s3 in slice_sum.items():
            p12 = np.einsum("ja,akc->jkc", g1[i1], g2[:, i2])          # [d1][d2][r2]
            out[b] += np.einsum("jkc,cm->jkm", p12, s3).reshape(-1)    # [d1][d2][d3]
        groups += len(slice_sum)
    return out, groups


def index_graph_edges(indices, offsets, rank, hot_thresh: int, max_group: int = 64, bag_cap: int = 256) -> dict:
    """Weighted co-occurrence edges of one batch (Section III-G, index-graph generation): a dict
    {(u, v): weight} with u < v, written as plain loops.

    Every lookup becomes the node max(rank[row], hot_thresh) - hot_thresh (frequency rank shifted by
    the hot threshold; node 0 = all hot rows, dropped).  A bag contributes every pair of its
    distinct nodes once; bags with more than `max_group` distinct nodes keep the `max_group`
    smallest, and only the first `bag_cap` lookups of a bag are looked at (both are limits of the
    job, not of the paper, which pairs everything).  weight = number of bags holding both ends.
    """
    import itertools
    idx, off = _i64(indices), _i64(offsets)
    rank = np.asarray(rank)
    edges = {}
    for b in range(off.size - 1):
        nodes = set()
        for i in idx[off[b]:off[b + 1]][:bag_cap]:
            if 0 <= i < rank.size:
                node = max(int(rank[i]), hot_thresh) - hot_thresh
                if node > 0:
                    nodes.add(node)
        kept = sorted(nodes)[:max_group]
        for u, v in itertools.combinations(kept, 2):
            edges[(u, v)] = edges.get((u, v), 0) + 1
    return edges
