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
        if input.dim() == 2:
            if offsets is not None:
                raise ValueError("offsets must be None for 2-D input")
            bags, length = input.shape
            offsets = torch.arange(0, (bags + 1) * length, length, dtype=torch.int64, device=input.device)
            return input.reshape(-1).contiguous(), offsets
        if input.dim() != 1 or offsets is None:
            raise ValueError("1-D input needs offsets")
        offsets = offsets.to(torch.int64)
        if not self.include_last_offset:  # the library takes CSR offsets of length bags + 1
            offsets = torch.cat([offsets, torch.full((1,), input.numel(), dtype=torch.int64, device=input.device)])
        return input.contiguous(), offsets.contiguous()

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


class TTEmbeddingBagCollection(torch.nn.Module):
    """The sparse side of a DLRM: one `TTEmbeddingBag` per categorical feature (Section IV: the TT
    tables replace the model's embedding tables one for one).

    tables    iterable of `TTEmbeddingBag`, or of keyword dicts for its constructor
    streams   number of side streams the tables are dealt to in forward (1: the current stream).
              Tables are independent and a table's kernels are short, so several streams let the
              GPU overlap them; autograd runs a table's backward on the stream of its forward.
    forward(inputs) takes one `(input, offsets)` pair (or a 2-D `input`) per table and returns the
    list of pooled outputs `[bags x embedding_dim]`, in table order.
    """

    def __init__(self, tables, streams: int = 1):
        super().__init__()
        self.tables = torch.nn.ModuleList(
            [t if isinstance(t, TTEmbeddingBag) else TTEmbeddingBag(**t) for t in tables])
        if streams < 1:
            raise ValueError("streams must be at least 1")
        self.num_streams = int(streams)
        self._side = None

    def forward(self, inputs):
        inputs = list(inputs)
        if len(inputs) != len(self.tables):
            raise ValueError("one input per table: got %d for %d tables" % (len(inputs), len(self.tables)))
        pairs = [x if isinstance(x, (tuple, list)) else (x, None) for x in inputs]
        if self.num_streams == 1:
            return [bag(inp, off) for bag, (inp, off) in zip(self.tables, pairs)]
        if self._side is None:
            self._side = [torch.cuda.Stream() for _ in range(self.num_streams)]
        cur = torch.cuda.current_stream()
        for s in self._side:
            s.wait_stream(cur)
        outs = []
        for i, (bag, (inp, off)) in enumerate(zip(self.tables, pairs)):
            with torch.cuda.stream(self._side[i % self.num_streams]):
                outs.append(bag(inp, off))
        for s in self._side:
            cur.wait_stream(s)
        for o in outs:
            o.record_stream(cur)
        return outs
