"""`torch.nn.EmbeddingBag`-style module over the TT embedding-bag library (sum pooling).

The paper presents its operator as a drop-in replacement for PyTorch's EmbeddingBag whose
trainable parameters are the TT cores (Sections III-A and IV, "compatible with PyTorch").  This
module only wires the C-ABI calls into autograd: the index reorder of the batch is built once in
forward and reused by backward (Sections III-C / III-E), every arithmetic step runs in the HIP
kernels, and there is no CPU fallback.

Two ways to train:
  * default: backward returns core-shaped gradients for the three parameters, so any
    torch.optim optimizer can be used;
  * `fused_sgd_lr=lr`: backward applies `G <- G - lr * dG` inside the backward kernels
    (Section III-F, fused TT-core update) and reports no gradient for the cores.

Two more forward routes of the library are selectable:
  * `forward_route="sample"`: sample-level reuse (Section III-B reuse equation) on top of the reuse
    buffer of prefix products -- same bag sums, one chain per (bag, prefix) group; backward is
    unchanged (it only needs the plan);
  * `bf16_inference()` / `forward_bf16(...)`: forward on bf16 copies of the cores with fp32
    accumulation, for inference (no gradient); the copies are refreshed on request.

`TTFusedEmbeddingBags` holds SEVERAL tables of equal column factors and ranks as one fused TT table
(cores side by side along the row-factor axis) and serves all of them with one reorder, one forward
and one backward: what a model with many small tables needs to fill the GPU.
"""
from __future__ import annotations

import torch

from . import binding


class _TTBagFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, core0, core1, core2, indices, offsets, module):
        table = module._table((core0, core1, core2))
        plan = binding.tt_index_reorder(table, indices, offsets)
        if module.forward_route == "sample":
            out = binding.tt_emb_bag_forward_sample(table, plan, offsets)
        else:
            out = binding.tt_emb_bag_forward(table, plan, indices, offsets)
        ctx.module, ctx.table, ctx.plan = module, table, plan
        ctx.save_for_backward(indices, offsets)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        indices, offsets = ctx.saved_tensors
        grad_out = grad_out.contiguous()
        if grad_out.dtype != torch.float32:
            raise TypeError("the TT embedding bag computes in float32")
        module = ctx.module
        if module.fused_sgd_lr is not None:
            binding.tt_emb_bag_backward_sgd(ctx.table, ctx.plan, indices, offsets, grad_out, module.fused_sgd_lr)
            return None, None, None, None, None, None
        dcores = binding.tt_emb_bag_backward(ctx.table, ctx.plan, indices, offsets, grad_out)
        return dcores[0], dcores[1], dcores[2], None, None, None


def _csr_offsets(input, offsets, include_last_offset):
    """torch.nn.EmbeddingBag's (input, offsets) conventions -> flat indices + CSR offsets (bags + 1)."""
    if input.dim() == 2:
        if offsets is not None:
            raise ValueError("offsets must be None for 2-D input")
        bags, length = input.shape
        offsets = torch.arange(0, (bags + 1) * length, length, dtype=torch.int64, device=input.device)
        return input.reshape(-1).contiguous(), offsets
    if input.dim() != 1 or offsets is None:
        raise ValueError("1-D input needs offsets")
    offsets = offsets.to(torch.int64)
    if not include_last_offset:  # the library takes CSR offsets of length bags + 1
        offsets = torch.cat([offsets, torch.full((1,), input.numel(), dtype=torch.int64, device=input.device)])
    return input.contiguous(), offsets.contiguous()


class TTEmbeddingBag(torch.nn.Module):
    """Sum-pooling embedding bag whose table of `num_embeddings x embedding_dim` is held as three
    TT cores `G_k[r_k][n_k][d_k][r_{k+1}]` (flat float32 parameters `core0..core2`).

    n, d     row / column factors: prod(n) >= num_embeddings, prod(d) == embedding_dim
    ranks    (R1, R2)
    forward(input, offsets=None) follows torch.nn.EmbeddingBag: 1-D `input` with `offsets`
    (bag starts; with include_last_offset the last entry is len(input)), or 2-D `input` whose rows
    are bags of equal length.  Not supported (raise): per_sample_weights, padding_idx, max_norm,
    modes other than "sum".
    """

    def __init__(self, num_embeddings: int, embedding_dim: int, n, d, ranks, mode: str = "sum",
                 include_last_offset: bool = False, init_row_std: float = 0.1, fused_sgd_lr=None,
                 forward_route: str = "batch", device="cuda", generator=None):
        super().__init__()
        if mode != "sum":
            raise NotImplementedError("only sum pooling is defined for the TT embedding bag")
        n, d, ranks = tuple(int(x) for x in n), tuple(int(x) for x in d), tuple(int(x) for x in ranks)
        if len(n) != 3 or len(d) != 3 or len(ranks) != 2:
            raise ValueError("three row factors, three column factors and two ranks are required")
        if d[0] * d[1] * d[2] != embedding_dim:
            raise ValueError("prod(d) must equal embedding_dim")
        if n[0] * n[1] * n[2] < num_embeddings:
            raise ValueError("prod(n) must be at least num_embeddings")
        self.num_embeddings, self.embedding_dim = int(num_embeddings), int(embedding_dim)
        self.n, self.d, self.r = n, d, (1, ranks[0], ranks[1], 1)
        self.include_last_offset = bool(include_last_offset)
        self.fused_sgd_lr = None if fused_sgd_lr is None else float(fused_sgd_lr)
        if forward_route not in ("batch", "sample"):
            raise ValueError("forward_route is 'batch' (each distinct row once, then a bag sum) or 'sample'")
        self.forward_route = forward_route
        self._bf16_cores = None
        # a row entry is a sum of R1*R2 products of three core entries: choose the core scale so that
        # the rows start with standard deviation `init_row_std`
        s = (init_row_std ** 2 / (ranks[0] * ranks[1])) ** (1.0 / 6.0)
        for k in range(3):
            numel = self.r[k] * n[k] * d[k] * self.r[k + 1]
            w = torch.empty(numel, dtype=torch.float32, device=device)
            w.normal_(0.0, s, generator=generator)
            self.register_parameter("core%d" % k, torch.nn.Parameter(w))

    def cores(self):
        return [self.core0, self.core1, self.core2]

    def _table(self, cores) -> binding.Table:
        return binding.Table(self.num_embeddings, self.n, self.d, self.r, [c.detach() for c in cores])

    def _bag_offsets(self, input, offsets):
        return _csr_offsets(input, offsets, self.include_last_offset)

    def forward(self, input, offsets=None, per_sample_weights=None):
        if per_sample_weights is not None:
            raise NotImplementedError("per_sample_weights are not defined for the TT embedding bag")
        if not input.is_cuda or not self.core0.is_cuda:
            raise RuntimeError("the TT embedding bag runs on the GPU only (there is no CPU path)")
        if input.dtype != torch.int64:
            input = input.to(torch.int64)
        indices, offsets = self._bag_offsets(input, offsets)
        return _TTBagFunction.apply(self.core0, self.core1, self.core2, indices, offsets, self)

    def bf16_inference(self):
        """(Re)build the bf16 copies of the cores that `forward_bf16` reads; call again after the cores
        have changed.  Only for shapes the matrix-core kernels serve (the library refuses others)."""
        self._bf16_cores = binding.tt_cores_to_bf16(self._table(self.cores()))
        return self

    @torch.no_grad()
    def forward_bf16(self, input, offsets=None):
        """Inference forward on the bf16 copies of the cores (fp32 accumulation); no autograd graph."""
        if self._bf16_cores is None:
            self.bf16_inference()
        if input.dtype != torch.int64:
            input = input.to(torch.int64)
        indices, offsets = self._bag_offsets(input, offsets)
        table = self._table(self.cores())
        plan = binding.tt_index_reorder(table, indices, offsets)
        return binding.tt_emb_bag_forward_bf16(table, self._bf16_cores, plan, offsets)

    def extra_repr(self) -> str:
        return "%d x %d, n=%s, d=%s, ranks=%s, %.1fx smaller than dense%s" % (
            self.num_embeddings, self.embedding_dim, self.n, self.d, self.r[1:3],
            self.num_embeddings * self.embedding_dim / float(sum(p.numel() for p in self.parameters())),
            ", fused SGD lr=%g" % self.fused_sgd_lr if self.fused_sgd_lr is not None else "")

    @staticmethod
    def near_cubic_factors(num_embeddings: int):
        """Three near-equal row factors whose product covers `num_embeddings`."""
        n3 = 1
        while n3 ** 3 < num_embeddings:
            n3 += 1
        n2 = 1
        while n2 * n2 * n3 < num_embeddings:
            n2 += 1
        n1 = max(1, -(-num_embeddings // (n2 * n3)))
        return (n1, n2, n3)


class TTFusedEmbeddingBags(torch.nn.Module):
    """Several sum-pooling embedding bags of one embedding_dim, one set of column factors `d` and one
    pair of ranks, held as ONE fused TT table: core k is `[r_k][sum of the tables' n_k][d_k][r_k+1]`
    and table t owns a range of the middle axis of every core.  A row of table t is the product of
    its own three slices (TT-matrix equation, Section II-B; index split per table, Section III-B), so
    outputs and gradients are those of the separate tables -- computed with one reorder, one forward
    and one backward for all of them.

    tables    list of `(num_embeddings, (n1, n2, n3))`; the sums of the row factors must keep the
              fused row count below 2^31 (split the tables over several modules otherwise:
              `binding.fusion_groups` deals them out)
    forward(inputs) takes one `(input, offsets)` pair (or a 2-D `input`) per table, as
    `TTEmbeddingBag.forward` does, and returns the list of pooled outputs in table order (views of
    one `[all bags x embedding_dim]` tensor).  `fused_sgd_lr` as for `TTEmbeddingBag`.
    """

    def __init__(self, tables, embedding_dim: int, d, ranks, include_last_offset: bool = False,
                 init_row_std: float = 0.1, fused_sgd_lr=None, device="cuda", generator=None):
        super().__init__()
        d, ranks = tuple(int(x) for x in d), tuple(int(x) for x in ranks)
        if len(d) != 3 or len(ranks) != 2 or d[0] * d[1] * d[2] != embedding_dim:
            raise ValueError("three column factors with prod(d) == embedding_dim and two ranks are required")
        tables = [(int(rows), tuple(int(x) for x in n)) for rows, n in tables]
        for rows, n in tables:
            if len(n) != 3 or n[0] * n[1] * n[2] < rows:
                raise ValueError("every table needs three row factors with prod(n) >= num_embeddings")
        self.tables, self.embedding_dim = tables, int(embedding_dim)
        self.d, self.r = d, (1, ranks[0], ranks[1], 1)
        self.include_last_offset = bool(include_last_offset)
        self.fused_sgd_lr = None if fused_sgd_lr is None else float(fused_sgd_lr)
        self.forward_route = "batch"
        self.n = tuple(sum(n[k] for _, n in tables) for k in range(3))
        self.num_embeddings = self.n[0] * self.n[1] * self.n[2]  # rows of the fused table
        if self.num_embeddings >= 2 ** 31 - 1:
            raise ValueError("the fused table would have 2^31 rows or more: fuse fewer tables")
        self._fused = None  # binding.FusedLayout, built on first use (it needs the library)
        s = (init_row_std ** 2 / (ranks[0] * ranks[1])) ** (1.0 / 6.0)
        for k in range(3):
            w = torch.empty(self.r[k] * self.n[k] * d[k] * self.r[k + 1], dtype=torch.float32, device=device)
            w.normal_(0.0, s, generator=generator)
            self.register_parameter("core%d" % k, torch.nn.Parameter(w))

    def cores(self):
        return [self.core0, self.core1, self.core2]

    def member_core(self, t: int, k: int, core=None):
        """Table t's part of fused core k (or of a tensor of its size, e.g. `.grad`): a strided view
        `[r_k][n_k(t)][d_k][r_k+1]`."""
        core = self.cores()[k] if core is None else core
        o = sum(n[k] for _, n in self.tables[:t])
        return core.view(self.r[k], self.n[k], self.d[k], self.r[k + 1])[:, o:o + self.tables[t][1][k]]

    def _table(self, cores) -> binding.Table:
        return binding.Table(self.num_embeddings, self.n, self.d, self.r, [c.detach() for c in cores])

    def forward(self, inputs):
        inputs = list(inputs)
        if len(inputs) != len(self.tables):
            raise ValueError("one input per table: got %d for %d tables" % (len(inputs), len(self.tables)))
        if not self.core0.is_cuda:
            raise RuntimeError("the TT embedding bag runs on the GPU only (there is no CPU path)")
        idx, off = [], []
        for x in inputs:
            inp, o = x if isinstance(x, (tuple, list)) else (x, None)
            if inp.dtype != torch.int64:
                inp = inp.to(torch.int64)
            i, o = _csr_offsets(inp, o, self.include_last_offset)
            idx.append(i)
            off.append(o)
        if self._fused is None:
            self._fused = binding.FusedLayout(self.tables)
        f_idx, f_off = self._fused.fuse_lookups(idx, off)
        out = _TTBagFunction.apply(self.core0, self.core1, self.core2, f_idx, f_off, self)
        return list(torch.split(out, [o.numel() - 1 for o in off]))

    def extra_repr(self) -> str:
        return "%d tables fused into %s rows x %d, d=%s, ranks=%s" % (
            len(self.tables), "x".join(str(x) for x in self.n), self.embedding_dim, self.d, self.r[1:3])


class TTEmbeddingBagCollection(torch.nn.Module):
    """The sparse side of a DLRM: one `TTEmbeddingBag` per categorical feature (Section IV: the TT
    tables replace the model's embedding tables one for one).

    tables    iterable of `TTEmbeddingBag`, or of keyword dicts for its constructor
    streams   number of side streams the tables are dealt to in forward (1: the current stream).
              Tables are independent and a table's kernels are short, so several streams let the
              GPU overlap them; autograd runs a table's backward on the stream of its forward.
    fuse      store tables of one family (same column factors, ranks, offset convention and update
              mode) as fused tables (`TTFusedEmbeddingBags`, dealt out by `binding.fusion_groups`) and
              serve each fused table with one set of launches.  The parameters are then the fused
              cores (`self.fused[g].core0..2`; `member_core` gives a table's part); the given tables'
              core values are copied in.  `fuse_groups`: number of fused tables per family (None: the
              fewest the limits allow).
    forward(inputs) takes one `(input, offsets)` pair (or a 2-D `input`) per table and returns the
    list of pooled outputs `[bags x embedding_dim]`, in table order.
    """

    def __init__(self, tables, streams: int = 1, fuse: bool = False, fuse_groups=None):
        super().__init__()
        tables = [t if isinstance(t, TTEmbeddingBag) else TTEmbeddingBag(**t) for t in tables]
        if streams < 1:
            raise ValueError("streams must be at least 1")
        self.num_streams = int(streams)
        self._side = None
        self.num_tables = len(tables)
        if not fuse:
            self.tables = torch.nn.ModuleList(tables)
            self.fused, self._where = None, None
            return
        self.tables = None
        families = {}
        for t, bag in enumerate(tables):
            key = (bag.d, bag.r, bag.include_last_offset, bag.fused_sgd_lr, bag.core0.device)
            families.setdefault(key, []).append(t)
        fused, where = [], [None] * len(tables)
        for (d, r, last, lr, dev), idxs in families.items():
            members = [(tables[t].num_embeddings, tables[t].n) for t in idxs]
            for part in binding.fusion_groups(members, groups=fuse_groups):
                m = TTFusedEmbeddingBags([members[p] for p in part], d[0] * d[1] * d[2], d, r[1:3],
                                         include_last_offset=last, fused_sgd_lr=lr, device=dev)
                with torch.no_grad():
                    for pos, p in enumerate(part):
                        src = tables[idxs[p]]
                        for k in range(3):
                            m.member_core(pos, k).copy_(src.cores()[k].view(r[k], src.n[k], d[k], r[k + 1]))
                        where[idxs[p]] = (len(fused), pos)
                fused.append(m)
        self.fused = torch.nn.ModuleList(fused)
        self._where = where

    def forward(self, inputs):
        inputs = list(inputs)
        if len(inputs) != self.num_tables:
            raise ValueError("one input per table: got %d for %d tables" % (len(inputs), self.num_tables))
        if self.fused is not None:
            per_group = [[None] * len(m.tables) for m in self.fused]
            for t, x in enumerate(inputs):
                gi, pos = self._where[t]
                per_group[gi][pos] = x
            units = [(m, xs) for m, xs in zip(self.fused, per_group)]
            run = lambda unit: unit[0](unit[1])
        else:
            pairs = [x if isinstance(x, (tuple, list)) else (x, None) for x in inputs]
            units = list(zip(self.tables, pairs))
            run = lambda unit: unit[0](unit[1][0], unit[1][1])
        if self.num_streams == 1:
            results = [run(u) for u in units]
        else:
            if self._side is None:
                self._side = [torch.cuda.Stream() for _ in range(self.num_streams)]
            cur = torch.cuda.current_stream()
            for s in self._side:
                s.wait_stream(cur)
            results = []
            for i, u in enumerate(units):
                with torch.cuda.stream(self._side[i % self.num_streams]):
                    results.append(run(u))
            for s in self._side:
                cur.wait_stream(s)
            for r in results:
                for o in (r if isinstance(r, list) else [r]):
                    o.record_stream(cur)
        if self.fused is None:
            return results
        return [results[gi][pos] for gi, pos in self._where]
