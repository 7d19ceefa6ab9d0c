"""Thin ctypes binding of libtt_emb.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/tt_emb.h; PyTorch is used here for device memory (tensors) and
streams.  There is no CPU fallback: if the library is missing or a call
returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtt_emb.so")

TT_OK = 0
TT_ERR_INVALID_ARG = -1
TT_ERR_SHAPE = -2
TT_ERR_WORKSPACE = -3
TT_ERR_INDEX_RANGE = -4
TT_ERR_HIP = -5
TT_ERR_UNAVAILABLE = -6

EXPORTS = ("tt_workspace_bytes", "tt_index_reorder", "tt_emb_bag_forward", "tt_emb_bag_backward",
           "tt_core_sgd_update", "tt_emb_bag_backward_sgd", "tt_emb_bag_forward_static", "tt_reuse_buffer_bytes", "tt_emb_bag_forward_sample",
           "tt_bf16_cores_bytes", "tt_cores_to_bf16", "tt_emb_bag_forward_bf16",
           "tt_index_graph_workspace_bytes", "tt_index_graph_edges", "tt_fuse_shape", "tt_fuse_lookups", "tt_plan_status", "tt_strerror", "tt_prof_create", "tt_prof_destroy",
           "tt_prof_collect", "tt_kernel_name", "tt_batch_desc_bytes", "tt_index_reorder_batched",
           "tt_emb_bag_forward_batched", "tt_emb_bag_backward_batched", "tt_core_sgd_update_batched")
KERNELS = {"fwd_contract": 0, "bag_sum": 1, "grad_merge": 2, "bwd_contract": 3, "sort_scatter": 4, "sgd": 5,
           "p12_fill": 6, "bag_chains": 7}


class TTError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, strerror(status), status))


class CTable(ctypes.Structure):
    _fields_ = [("num_rows", ctypes.c_int64), ("n", ctypes.c_int32 * 3), ("d", ctypes.c_int32 * 3),
                ("r", ctypes.c_int32 * 4), ("core", ctypes.c_void_p * 3)]


_I32P = ctypes.c_void_p
_PLAN_INT_ARRAYS = ("sorted_row", "perm", "bag_of_sorted", "slot_of_sorted", "lookup2row", "uniq_row",
                    "row_seg", "row2pref", "uniq_pref", "pref_seg", "rows_by_i3", "i3_of_sorted",
                    "i3_seg", "prefs_by_i2", "i2_seg", "i1_seg", "pref_meta", "counts")
_PLAN_FLOAT_ARRAYS = ("rowbuf", "gagg", "hbuf", "t3buf", "t1buf", "partial", "dg2part")


class CPlan(ctypes.Structure):
    _fields_ = ([("nnz", ctypes.c_int64), ("num_bags", ctypes.c_int64), ("max_rows", ctypes.c_int64),
                 ("max_prefixes", ctypes.c_int64), ("n", ctypes.c_int32 * 3), ("d", ctypes.c_int32 * 3),
                 ("r", ctypes.c_int32 * 4)]
                + [(name, _I32P) for name in _PLAN_INT_ARRAYS]
                + [(name, ctypes.c_void_p) for name in _PLAN_FLOAT_ARRAYS]
                + [("sort_tmp", ctypes.c_void_p), ("prof", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                   ("workspace_bytes", ctypes.c_size_t)])


class CBatchItem(ctypes.Structure):
    _fields_ = [("table", ctypes.c_void_p), ("plan", ctypes.c_void_p), ("indices", ctypes.c_void_p),
                ("offsets", ctypes.c_void_p), ("nnz", ctypes.c_int64), ("num_bags", ctypes.c_int64),
                ("remap", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("out", ctypes.c_void_p),
                ("grad_out", ctypes.c_void_p), ("dcore", ctypes.c_void_p * 3)]


TT_FUSE_MAX_TABLES = 32


class CFuseMembers(ctypes.Structure):
    _fields_ = [("num_tables", ctypes.c_int32), ("n", (ctypes.c_int32 * 3) * TT_FUSE_MAX_TABLES),
                ("num_rows", ctypes.c_int64 * TT_FUSE_MAX_TABLES)]


_lib = None


def load_library():
    """Load libtt_emb.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(hipcc, gfx950) first; there is no fallback path" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float
        lib.tt_workspace_bytes.restype = ctypes.c_size_t
        lib.tt_workspace_bytes.argtypes = [vp, i64, i64]
        lib.tt_index_reorder.restype = ctypes.c_int
        lib.tt_index_reorder.argtypes = [vp, vp, vp, i64, i64, vp, vp, ctypes.c_size_t, vp, vp]
        lib.tt_emb_bag_forward.restype = ctypes.c_int
        lib.tt_emb_bag_forward.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp]
        lib.tt_emb_bag_backward.restype = ctypes.c_int
        lib.tt_emb_bag_backward.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp]
        lib.tt_core_sgd_update.restype = ctypes.c_int
        lib.tt_core_sgd_update.argtypes = [vp, vp, vp, f32, vp]
        lib.tt_emb_bag_backward_sgd.restype = ctypes.c_int
        lib.tt_emb_bag_backward_sgd.argtypes = [vp, vp, vp, vp, i64, i64, vp, f32, vp]
        lib.tt_emb_bag_forward_static.restype = ctypes.c_int
        lib.tt_emb_bag_forward_static.argtypes = [vp, vp, vp, i64, i64, vp, vp]
        lib.tt_reuse_buffer_bytes.restype = ctypes.c_size_t
        lib.tt_reuse_buffer_bytes.argtypes = [vp, i64]
        lib.tt_emb_bag_forward_sample.restype = ctypes.c_int
        lib.tt_emb_bag_forward_sample.argtypes = [vp, vp, vp, i64, i64, vp, ctypes.c_size_t, vp, vp]
        lib.tt_bf16_cores_bytes.restype = ctypes.c_size_t
        lib.tt_bf16_cores_bytes.argtypes = [vp]
        lib.tt_cores_to_bf16.restype = ctypes.c_int
        lib.tt_cores_to_bf16.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.tt_emb_bag_forward_bf16.restype = ctypes.c_int
        lib.tt_emb_bag_forward_bf16.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp]
        lib.tt_index_graph_workspace_bytes.restype = ctypes.c_size_t
        lib.tt_index_graph_workspace_bytes.argtypes = [i64, i64]
        lib.tt_index_graph_edges.restype = ctypes.c_int
        lib.tt_index_graph_edges.argtypes = [vp, vp, i64, i64, vp, i64, i64, ctypes.c_int32, vp, ctypes.c_size_t, i64,
                                             vp, vp, vp, vp, vp]
        lib.tt_fuse_shape.restype = ctypes.c_int
        lib.tt_fuse_shape.argtypes = [vp, vp]
        lib.tt_fuse_lookups.restype = ctypes.c_int
        lib.tt_fuse_lookups.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.tt_plan_status.restype = ctypes.c_int
        lib.tt_plan_status.argtypes = [vp, vp, vp]
        lib.tt_prof_create.restype = vp
        lib.tt_prof_create.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.tt_prof_destroy.restype = None
        lib.tt_prof_destroy.argtypes = [vp]
        lib.tt_prof_collect.restype = ctypes.c_int
        lib.tt_prof_collect.argtypes = [vp, vp, vp]
        lib.tt_kernel_name.restype = ctypes.c_char_p
        lib.tt_kernel_name.argtypes = [ctypes.c_int]
        lib.tt_strerror.restype = ctypes.c_char_p
        lib.tt_strerror.argtypes = [ctypes.c_int]
        lib.tt_batch_desc_bytes.restype = ctypes.c_size_t
        lib.tt_batch_desc_bytes.argtypes = [ctypes.c_int]
        for name in ("tt_index_reorder_batched", "tt_emb_bag_forward_batched", "tt_emb_bag_backward_batched"):
            f = getattr(lib, name)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_int, vp, vp, ctypes.c_size_t, vp]
        lib.tt_core_sgd_update_batched.restype = ctypes.c_int
        lib.tt_core_sgd_update_batched.argtypes = [ctypes.c_int, vp, f32, vp, ctypes.c_size_t, vp]
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load_library().tt_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != TT_OK:
        raise TTError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev_i64(t, name):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.int64 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA int64 tensor" % name)
    return t


def _dev_f32(t, name):
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA float32 tensor" % name)
    return t


class Table:
    """A TT table: shape + three device-resident fp32 cores (flat, [r][n][d][r'] order)."""

    def __init__(self, num_rows, n, d, r, cores):
        self.num_rows, self.n, self.d, self.r = int(num_rows), tuple(n), tuple(d), tuple(r)
        self.cores = [_dev_f32(c, "core") for c in cores]
        for k in range(3):
            want = self.r[k] * self.n[k] * self.d[k] * self.r[k + 1]
            if self.cores[k].numel() != want:
                raise ValueError("core %d has %d elements, expected %d" % (k, self.cores[k].numel(), want))
        self.dim = self.d[0] * self.d[1] * self.d[2]
        c = CTable()
        c.num_rows = self.num_rows
        c.n[:] = self.n
        c.d[:] = self.d
        c.r[:] = self.r
        for k in range(3):
            c.core[k] = self.cores[k].data_ptr()
        self.c = c

    @classmethod
    def from_numpy(cls, shape, cores, device="cuda"):
        return cls(shape.num_rows, shape.n, shape.d, shape.r,
                   [torch.from_numpy(c).to(device).contiguous() for c in cores])

    def core_grads_like(self):
        return [torch.empty_like(c) for c in self.cores]


class Plan:
    """Host view of a reorder plan; owns (or borrows) the device workspace tensor."""

    def __init__(self, workspace):
        self.workspace = workspace
        self.c = CPlan()

    def _array(self, name, count, dtype):
        addr = getattr(self.c, name)
        off = addr - self.workspace.data_ptr()
        esz = 4
        return self.workspace[off:off + count * esz].view(dtype)

    def counts(self, stream=None):
        """(U_r, U_p, valid lookups, status bits); synchronises the stream."""
        out = (ctypes.c_int64 * 4)()
        st = load_library().tt_plan_status(ctypes.byref(self.c), _stream(stream), out)
        return tuple(int(x) for x in out), st

    def arrays(self, stream=None) -> dict:
        """Copies of the plan's index arrays trimmed to their valid lengths (test helper)."""
        (ur, up, nvalid, _), _ = self.counts(stream)
        nnz = int(self.c.nnz)
        lens = dict(sorted_row=nnz, perm=nnz, bag_of_sorted=nnz, slot_of_sorted=nnz, lookup2row=nnz,
                    uniq_row=ur, row_seg=ur + 1, row2pref=ur, uniq_pref=up, pref_seg=up + 1,
                    rows_by_i3=ur, i3_of_sorted=ur, i3_seg=self.c.n[2] + 1, prefs_by_i2=up,
                    i2_seg=self.c.n[1] + 1, i1_seg=self.c.n[0] + 1)
        out = {k: self._array(k, v, torch.int32).cpu().numpy() for k, v in lens.items()}
        out.update(U_r=ur, U_p=up, num_valid=nvalid)
        return out


class Prof:
    """HIP-event timing of one kernel of the planned path (benchmark helper)."""

    def __init__(self, kernel: str, capacity: int):
        self.kernel = kernel
        self.handle = load_library().tt_prof_create(KERNELS[kernel], int(capacity))
        if not self.handle:
            raise TTError(TT_ERR_HIP, "tt_prof_create")

    def attach(self, plan: "Plan"):
        plan.c.prof = self.handle

    def collect(self):
        """(total milliseconds, launches) since the last collect; waits for the events."""
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(load_library().tt_prof_collect(self.handle, ctypes.byref(ms), ctypes.byref(n)), "tt_prof_collect")
        return ms.value, n.value

    def close(self):
        if self.handle:
            load_library().tt_prof_destroy(self.handle)
            self.handle = None


def tt_workspace_bytes(table: Table, nnz: int, num_bags: int) -> int:
    return int(load_library().tt_workspace_bytes(ctypes.byref(table.c), int(nnz), int(num_bags)))


def alloc_workspace(table: Table, nnz: int, num_bags: int, device="cuda"):
    nbytes = tt_workspace_bytes(table, nnz, num_bags)
    if nbytes == 0:
        raise TTError(TT_ERR_SHAPE, "tt_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def tt_index_reorder(table: Table, indices, offsets, remap=None, workspace=None, stream=None) -> Plan:
    indices, offsets = _dev_i64(indices, "indices"), _dev_i64(offsets, "offsets")
    remap = _dev_i64(remap, "remap")
    nnz, nb = indices.numel(), offsets.numel() - 1
    if workspace is None:
        workspace = alloc_workspace(table, nnz, nb, indices.device)
    plan = Plan(workspace)
    st = load_library().tt_index_reorder(ctypes.byref(table.c), _ptr(indices), _ptr(offsets), nnz, nb,
                                         _ptr(remap), _ptr(workspace), workspace.numel(),
                                         ctypes.byref(plan.c), _stream(stream))
    _check(st, "tt_index_reorder")
    return plan


def tt_emb_bag_forward(table: Table, plan, indices, offsets, out=None, stream=None):
    indices, offsets = _dev_i64(indices, "indices"), _dev_i64(offsets, "offsets")
    nnz, nb = indices.numel(), offsets.numel() - 1
    if out is None:
        out = torch.empty((nb, table.dim), dtype=torch.float32, device=offsets.device)
    _dev_f32(out, "out")
    st = load_library().tt_emb_bag_forward(ctypes.byref(table.c), ctypes.byref(plan.c) if plan else None,
                                           _ptr(indices), _ptr(offsets), nnz, nb, _ptr(out), _stream(stream))
    _check(st, "tt_emb_bag_forward")
    return out


def tt_reuse_buffer_bytes(table: Table, nnz: int) -> int:
    return int(load_library().tt_reuse_buffer_bytes(ctypes.byref(table.c), int(nnz)))


def tt_emb_bag_forward_sample(table: Table, plan, offsets, reuse_buffer=None, out=None, stream=None):
    """Forward by sample-level reuse: reuse buffer of prefix products, then one chain per (bag, prefix)."""
    offsets = _dev_i64(offsets, "offsets")
    nnz, nb = int(plan.c.nnz), offsets.numel() - 1
    if reuse_buffer is None:
        reuse_buffer = torch.empty(tt_reuse_buffer_bytes(table, nnz), dtype=torch.uint8, device=offsets.device)
    if out is None:
        out = torch.empty((nb, table.dim), dtype=torch.float32, device=offsets.device)
    _dev_f32(out, "out")
    st = load_library().tt_emb_bag_forward_sample(ctypes.byref(table.c), ctypes.byref(plan.c), _ptr(offsets), nnz, nb,
                                                  _ptr(reuse_buffer), reuse_buffer.numel(), _ptr(out), _stream(stream))
    _check(st, "tt_emb_bag_forward_sample")
    return out


def tt_index_graph_edges(indices, offsets, rank, hot_thresh: int, max_group: int = 64, max_pairs: int = None,
                         stream=None):
    """Co-occurrence edges of one batch on the GPU: (u, v, w) int32 device tensors sorted by (u, v).
    Synchronises to read the edge count.  `rank` is an int32 device tensor of frequency ranks."""
    indices, offsets = _dev_i64(indices, "indices"), _dev_i64(offsets, "offsets")
    if rank.dtype != torch.int32 or not rank.is_cuda or not rank.is_contiguous():
        raise TypeError("rank must be a contiguous int32 device tensor")
    nnz, nb = indices.numel(), offsets.numel() - 1
    if max_pairs is None:  # every bag pairs at most min(length, max_group) nodes
        lens = torch.clamp(offsets[1:] - offsets[:-1], max=max_group)
        max_pairs = max(1, int((lens * (lens - 1) // 2).sum().item()))
    lib = load_library()
    ws = torch.empty(lib.tt_index_graph_workspace_bytes(nb, max_pairs), dtype=torch.uint8, device=indices.device)
    eu, ev, ew = (torch.empty(max_pairs, dtype=torch.int32, device=indices.device) for _ in range(3))
    counts = torch.zeros(4, dtype=torch.int32, device=indices.device)
    st = lib.tt_index_graph_edges(_ptr(indices), _ptr(offsets), nnz, nb, _ptr(rank), rank.numel(), int(hot_thresh),
                                  int(max_group), _ptr(ws), ws.numel(), max_pairs, _ptr(eu), _ptr(ev), _ptr(ew),
                                  _ptr(counts), _stream(stream))
    _check(st, "tt_index_graph_edges")
    c = counts.cpu().tolist()  # synchronises
    if c[2] != 0:
        raise TTError(TT_ERR_WORKSPACE, "tt_index_graph_edges: more pairs than max_pairs")
    return eu[:c[1]], ev[:c[1]], ew[:c[1]]


def tt_bf16_cores_bytes(table: Table) -> int:
    return int(load_library().tt_bf16_cores_bytes(ctypes.byref(table.c)))


def tt_cores_to_bf16(table: Table, bf16_cores=None, stream=None):
    """bf16 copies of the table's cores (library-private layout) in a uint8 device tensor."""
    nbytes = tt_bf16_cores_bytes(table)
    if nbytes == 0:
        raise TTError(TT_ERR_SHAPE, "tt_bf16_cores_bytes")
    if bf16_cores is None:
        bf16_cores = torch.empty(nbytes, dtype=torch.uint8, device=table.cores[0].device)
    st = load_library().tt_cores_to_bf16(ctypes.byref(table.c), _ptr(bf16_cores), bf16_cores.numel(), _stream(stream))
    _check(st, "tt_cores_to_bf16")
    return bf16_cores


def tt_emb_bag_forward_bf16(table: Table, bf16_cores, plan, offsets, out=None, stream=None):
    offsets = _dev_i64(offsets, "offsets")
    nnz, nb = int(plan.c.nnz), offsets.numel() - 1
    if out is None:
        out = torch.empty((nb, table.dim), dtype=torch.float32, device=offsets.device)
    _dev_f32(out, "out")
    st = load_library().tt_emb_bag_forward_bf16(ctypes.byref(table.c), _ptr(bf16_cores), ctypes.byref(plan.c),
                                                _ptr(offsets), nnz, nb, _ptr(out), _stream(stream))
    _check(st, "tt_emb_bag_forward_bf16")
    return out


def tt_emb_bag_forward_static(table: Table, indices, offsets, out, stream=None):
    """Reorder + planned forward in the library's static scratch: allocates nothing (`out` is required)."""
    indices, offsets = _dev_i64(indices, "indices"), _dev_i64(offsets, "offsets")
    _dev_f32(out, "out")
    nnz, nb = indices.numel(), offsets.numel() - 1
    if out.numel() != nb * table.dim:
        raise ValueError("out must hold num_bags * D floats")
    st = load_library().tt_emb_bag_forward_static(ctypes.byref(table.c), _ptr(indices), _ptr(offsets), nnz, nb,
                                                  _ptr(out), _stream(stream))
    _check(st, "tt_emb_bag_forward_static")
    return out


def tt_emb_bag_backward(table: Table, plan, indices, offsets, grad_out, dcores=None, stream=None):
    indices, offsets = _dev_i64(indices, "indices"), _dev_i64(offsets, "offsets")
    _dev_f32(grad_out, "grad_out")
    nnz, nb = indices.numel(), offsets.numel() - 1
    if grad_out.numel() != nb * table.dim:
        raise ValueError("grad_out must hold num_bags * D floats")
    if dcores is None:
        dcores = table.core_grads_like()
    arr = (ctypes.c_void_p * 3)(*[_dev_f32(g, "dcore").data_ptr() for g in dcores])
    st = load_library().tt_emb_bag_backward(ctypes.byref(table.c), ctypes.byref(plan.c) if plan else None,
                                            _ptr(indices), _ptr(offsets), nnz, nb, _ptr(grad_out), arr,
                                            _stream(stream))
    _check(st, "tt_emb_bag_backward")
    return dcores


def tt_emb_bag_backward_sgd(table: Table, plan: Plan, indices, offsets, grad_out, lr: float, stream=None):
    """Backward with the core update fused in: the table's cores are updated in place."""
    indices, offsets = _dev_i64(indices, "indices"), _dev_i64(offsets, "offsets")
    _dev_f32(grad_out, "grad_out")
    nnz, nb = indices.numel(), offsets.numel() - 1
    if grad_out.numel() != nb * table.dim:
        raise ValueError("grad_out must hold num_bags * D floats")
    st = load_library().tt_emb_bag_backward_sgd(ctypes.byref(table.c), ctypes.byref(plan.c) if plan else None,
                                                _ptr(indices), _ptr(offsets), nnz, nb, _ptr(grad_out),
                                                ctypes.c_float(lr), _stream(stream))
    _check(st, "tt_emb_bag_backward_sgd")


def tt_core_sgd_update(table: Table, plan, dcores, lr: float, stream=None):
    arr = (ctypes.c_void_p * 3)(*[_dev_f32(g, "dcore").data_ptr() for g in dcores])
    st = load_library().tt_core_sgd_update(ctypes.byref(table.c), ctypes.byref(plan.c) if plan else None,
                                           arr, ctypes.c_float(lr), _stream(stream))
    _check(st, "tt_core_sgd_update")


def tt_plan_status(plan: Plan, stream=None) -> int:
    _, st = plan.counts(stream)
    return st


# ------------------------------------------------------------------ fused tables
class FusedLayout:
    """Index space of several TT tables stored as one: `members` is a list of `(num_rows, (n1, n2, n3))`;
    `n` are the fused row factors, `start[t][k]` member t's first index in fused core k.
    `fuse_lookups` maps one batch of every member into the fused table; rows of the fused `out` /
    `grad_out` are the members' bags, member after member (`bag_ranges`)."""

    def __init__(self, members):
        members = [(int(nr), tuple(int(x) for x in n)) for nr, n in members]
        if not 1 <= len(members) <= TT_FUSE_MAX_TABLES:
            raise ValueError("1 to %d member tables" % TT_FUSE_MAX_TABLES)
        self.members = members
        c = CFuseMembers()
        c.num_tables = len(members)
        for t, (nr, n) in enumerate(members):
            c.n[t][:] = n
            c.num_rows[t] = nr
        self.c = c
        shape = CTable()
        _check(load_library().tt_fuse_shape(ctypes.byref(c), ctypes.byref(shape)), "tt_fuse_shape")
        self.n, self.num_rows = tuple(shape.n), int(shape.num_rows)
        self.start = [[sum(m[1][k] for m in members[:t]) for k in range(3)] for t in range(len(members))]

    def bag_ranges(self, num_bags):
        out, b0 = [], 0
        for nb in num_bags:
            out.append((b0, b0 + int(nb)))
            b0 += int(nb)
        return out

    def fuse_lookups(self, indices, offsets, remaps=None, out=None, stream=None):
        """Maps the members' `(indices[t], offsets[t])` (CSR offsets, `bags + 1` long) into the fused
        table: returns `(fused_indices, fused_offsets)`; `out` may bring the two tensors to write."""
        T = len(self.members)
        if len(indices) != T or len(offsets) != T:
            raise ValueError("one (indices, offsets) pair per member table")
        idx = [_dev_i64(x, "indices") for x in indices]
        off = [_dev_i64(x, "offsets") for x in offsets]
        rm = [None] * T if remaps is None else [_dev_i64(x, "remap") for x in remaps]
        nnz = [x.numel() for x in idx]
        nb = [x.numel() - 1 for x in off]
        dev = off[0].device
        if out is None:
            out = (torch.empty(sum(nnz), dtype=torch.int64, device=dev),
                   torch.empty(sum(nb) + 1, dtype=torch.int64, device=dev))
        f_idx, f_off = _dev_i64(out[0], "fused_indices"), _dev_i64(out[1], "fused_offsets")
        if f_idx.numel() != sum(nnz) or f_off.numel() != sum(nb) + 1:
            raise ValueError("fused_indices / fused_offsets have the wrong length")
        ptrs = lambda ts: (ctypes.c_void_p * T)(*[None if x is None or x.numel() == 0 else x.data_ptr() for x in ts])
        i64s = lambda vs: (ctypes.c_int64 * T)(*vs)
        st = load_library().tt_fuse_lookups(ctypes.byref(self.c), ptrs(idx), ptrs(off), ptrs(rm) if remaps is not None else None,
                                            i64s(nnz), i64s(nb), _ptr(f_idx), _ptr(f_off), _stream(stream))
        _check(st, "tt_fuse_lookups")
        return f_idx, f_off


class FusedTables(FusedLayout):
    """Several TT tables with equal column factors and ranks stored as ONE table: core k of the fused
    table is `[r_k][sum of the members' n_k][d_k][r_k+1]`, member t owning a range of the middle axis.

    members   list of `(num_rows, (n1, n2, n3))`
    cores     optional list (per member) of three flat fp32 tensors / arrays to start from; without
              it the fused cores are zero and left for the caller to fill (`member_core` gives the views)
    `table` is the fused `Table` that every single-table call of this module takes.
    """

    def __init__(self, members, d, r, cores=None, device="cuda"):
        super().__init__(members)
        self.d, self.r = tuple(d), tuple(r)
        members = self.members
        fused = [torch.zeros(self.r[k] * self.n[k] * self.d[k] * self.r[k + 1], dtype=torch.float32, device=device)
                 for k in range(3)]
        self.table = Table(self.num_rows, self.n, self.d, self.r, fused)
        if cores is not None:
            for t in range(len(members)):
                for k in range(3):
                    src = torch.as_tensor(cores[t][k]).to(device=device, dtype=torch.float32)
                    self.member_core(t, k).copy_(src.view(self.r[k], members[t][1][k], self.d[k], self.r[k + 1]))

    def core_view(self, k, core=None):
        """Core k of the fused table (or a tensor of its size, e.g. a gradient) as `[r_k][N_k][d_k][r_k+1]`."""
        core = self.table.cores[k] if core is None else core
        return core.view(self.r[k], self.n[k], self.d[k], self.r[k + 1])

    def member_core(self, t, k, core=None):
        """Member t's part of (a tensor shaped like) fused core k: a strided view `[r_k][n_k(t)][d_k][r_k+1]`."""
        o = self.start[t][k]
        return self.core_view(k, core)[:, o:o + self.members[t][1][k]]


def fusion_groups(members, groups=None, max_factor_sum=1023):
    """Deals tables to fused groups: `members` is a list of `(num_rows, n)`; returns lists of member
    positions, largest member first.  Largest tables first, each into the group with the smallest sum of row factors so
    far; `groups=None` takes the fewest groups whose factor sums stay within `max_factor_sum` (1023
    keeps every grouping of the reorder a single radix digit) and whose rows stay below 2^31."""
    order = sorted(range(len(members)), key=lambda t: -max(members[t][1]))
    g = max(1, groups or 1)
    while True:
        parts, sums = [[] for _ in range(g)], [[0, 0, 0] for _ in range(g)]
        for t in order:
            k = min(range(g), key=lambda j: max(sums[j]))
            parts[k].append(t)
            for a in range(3):
                sums[k][a] += members[t][1][a]
        ok = all(max(sm) <= max_factor_sum and sm[0] * sm[1] * sm[2] < 2 ** 31 - 1 and len(p) <= TT_FUSE_MAX_TABLES
                 for sm, p in zip(sums, parts) if p)
        if ok or g >= len(members):
            if not ok:
                raise ValueError("no fusion of these tables fits the limits")
            return [p for p in parts if p]  # largest member first: its long-running workgroups start early
        g += 1


# ------------------------------------------------------------------ batched calls
def alloc_batch_desc(num_tables: int, device="cuda"):
    """Device scratch for the per-table kernel descriptors of ONE batched call in flight."""
    nbytes = int(load_library().tt_batch_desc_bytes(int(num_tables)))
    if nbytes == 0:
        raise TTError(TT_ERR_INVALID_ARG, "tt_batch_desc_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _items(tables, plans=None, indices=None, offsets=None, remaps=None, workspaces=None, outs=None,
           grads=None, dcores=None):
    n = len(tables)
    arr = (CBatchItem * n)()
    for t in range(n):
        it = arr[t]
        it.table = ctypes.addressof(tables[t].c)
        if plans is not None and plans[t] is not None:
            it.plan = ctypes.addressof(plans[t].c)
        if indices is not None:
            it.indices = _dev_i64(indices[t], "indices").data_ptr()
            it.nnz = indices[t].numel()
        if offsets is not None:
            it.offsets = _dev_i64(offsets[t], "offsets").data_ptr()
            it.num_bags = offsets[t].numel() - 1
        if remaps is not None and remaps[t] is not None:
            it.remap = _dev_i64(remaps[t], "remap").data_ptr()
        if workspaces is not None:
            it.workspace = workspaces[t].data_ptr()
            it.workspace_bytes = workspaces[t].numel()
        if outs is not None:
            it.out = _dev_f32(outs[t], "out").data_ptr()
        if grads is not None:
            it.grad_out = _dev_f32(grads[t], "grad_out").data_ptr()
        if dcores is not None:
            for k in range(3):
                it.dcore[k] = _dev_f32(dcores[t][k], "dcore").data_ptr()
    return arr


def tt_index_reorder_batched(tables, indices, offsets, workspaces, desc, remaps=None, stream=None):
    """One reorder plan per table, built with one launch per kernel for the whole batch."""
    plans = [Plan(ws) for ws in workspaces]
    arr = _items(tables, plans, indices, offsets, remaps, workspaces)
    st = load_library().tt_index_reorder_batched(len(tables), arr, _ptr(desc), desc.numel(), _stream(stream))
    _check(st, "tt_index_reorder_batched")
    return plans


def tt_emb_bag_forward_batched(tables, plans, indices, offsets, outs, desc, stream=None):
    arr = _items(tables, plans, indices, offsets, outs=outs)
    st = load_library().tt_emb_bag_forward_batched(len(tables), arr, _ptr(desc), desc.numel(), _stream(stream))
    _check(st, "tt_emb_bag_forward_batched")
    return outs


def tt_emb_bag_backward_batched(tables, plans, indices, offsets, grads, dcores, desc, stream=None):
    arr = _items(tables, plans, indices, offsets, grads=grads, dcores=dcores)
    st = load_library().tt_emb_bag_backward_batched(len(tables), arr, _ptr(desc), desc.numel(), _stream(stream))
    _check(st, "tt_emb_bag_backward_batched")
    return dcores


def tt_core_sgd_update_batched(tables, plans, dcores, lr, desc, stream=None):
    arr = _items(tables, plans, dcores=dcores)
    st = load_library().tt_core_sgd_update_batched(len(tables), arr, ctypes.c_float(lr), _ptr(desc),
                                                   desc.numel(), _stream(stream))
    _check(st, "tt_core_sgd_update_batched")
