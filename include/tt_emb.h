/*
 * tt_emb.h -- C ABI of the Tensor-Train (TT) embedding-bag hot path for MI355X (gfx950).
 *
 * The operator is an nn.EmbeddingBag-style lookup (flat index list + CSR bag
 * offsets, sum pooling) whose trainable parameters are three TT cores (paper,
 * Section II-B; Section III-A..F for the optimised lookup / backward).
 *
 * Conventions shared by every call
 * --------------------------------
 * - "DEVICE" pointers are HIP device memory of the current device; "HOST"
 *   pointers are ordinary host memory.  The library allocates no device memory:
 *   every buffer, including the workspace a plan lives in, is owned by the caller
 *   and merely borrowed until the work enqueued by the call has finished on
 *   `stream`.  The only process-wide state is a once-per-process set-up of kernel
 *   launch attributes (thread-safe); calls may be issued from several host threads.
 * - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *   default stream).  No call synchronises or copies device->host, except
 *   tt_plan_status.
 * - Core k (k = 0,1,2) is a flat fp32 array indexed G_k[r[k]][n[k]][d[k]][r[k+1]],
 *   row-major, with r[0] = r[3] = 1 (Section II-B: boundary ranks are 1).
 *   A table has num_rows <= n[0]*n[1]*n[2] rows; rows >= num_rows are padding
 *   and are never valid.  Row i uses slices (i1,i2,i3) with
 *   i3 = i mod n[2], i2 = (i div n[2]) mod n[1], i1 = i div (n[1]*n[2])
 *   (Section III-B, TT-index equation; i1 is the most significant digit), and
 *   its D = d[0]*d[1]*d[2] columns are ordered j = (j1*d[1] + j2)*d[2] + j3.
 * - Bags are CSR: offsets has num_bags+1 entries, offsets[0] = 0,
 *   offsets[num_bags] = nnz, non-decreasing.  An empty bag gives a zero row.
 *   Indices and offsets are int64 (the PyTorch default); everything else fp32.
 * - Every call returns a tt_status and never throws.  Host-visible arguments
 *   (NULL pointers, shapes, sizes) are validated synchronously.  Errors only
 *   the device can see (an index < 0 or >= num_rows, offsets that are not
 *   monotone) set a status word inside the plan; the offending lookup then
 *   contributes nothing, and tt_plan_status reports it.  Without a plan
 *   (naive arms) an out-of-range lookup is skipped silently.
 * - With a plan every result is bitwise reproducible from run to run (sorted
 *   segmented reductions, no floating-point atomics).  The plan == NULL
 *   backward accumulates with floating-point atomics and is not.
 * - Limits (TT_ERR_SHAPE otherwise): n[0]*n[1]*n[2] < 2^31 - 1, nnz < 2^31 - 1,
 *   r[1], r[2] <= 128, d[0]*d[1]*r[2] <= 4096, d[1]*r[2] <= 4096, D <= 1024.
 */
#ifndef TT_EMB_H_
#define TT_EMB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TT_OK = 0,
  TT_ERR_INVALID_ARG = -1, /* NULL pointer, negative size                                */
  TT_ERR_SHAPE = -2,       /* table shape violates the conventions or limits above       */
  TT_ERR_WORKSPACE = -3,   /* workspace too small or misaligned (needs 256-byte align)   */
  TT_ERR_INDEX_RANGE = -4, /* reported by tt_plan_status: bad index or bad offsets seen  */
  TT_ERR_HIP = -5,         /* a HIP runtime call or kernel launch failed                 */
  TT_ERR_UNAVAILABLE = -6  /* the entry point is switched off in this build              */
} tt_status;

/* One TT table.  HOST struct, caller-owned, read during the call only. */
typedef struct {
  int64_t num_rows; /* N, number of valid rows                                         */
  int32_t n[3];     /* row factors, n[0]*n[1]*n[2] >= N                                */
  int32_t d[3];     /* column factors, D = d[0]*d[1]*d[2]                              */
  int32_t r[4];     /* TT ranks, r[0] = r[3] = 1                                       */
  float *core[3];   /* DEVICE, core k is [r[k]][n[k]][d[k]][r[k+1]] row-major          */
} tt_table;

/*
 * The reorder plan: a HOST struct of DEVICE pointers into the caller's
 * workspace, filled by tt_index_reorder.  It is the deterministic counterpart
 * of the paper's reuse-buffer bookkeeping (Section III-C, pointer-preparation
 * algorithm) and of the "distinct embeddings" bookkeeping of the gradient
 * aggregation (Section III-E): lookups stably sorted by row, the distinct rows,
 * and the distinct (i1,i2) prefixes (prefix = row div n[2], the reuse-buffer
 * key), each in increasing order.  U_r = number of distinct valid rows, U_p =
 * number of distinct prefixes; both live on the device (counts[0], counts[1]).
 * All index arrays are int32.  Entries beyond the stated valid length are
 * unspecified.  The same plan serves forward, backward and update of the batch
 * it was built from, for this table shape only.
 */
typedef struct {
  int64_t nnz, num_bags;  /* the batch the plan was built for                            */
  int64_t max_rows;       /* capacity for distinct rows     = min(nnz, num_rows)          */
  int64_t max_prefixes;   /* capacity for distinct prefixes = min(nnz, n[0]*n[1])         */
  int32_t n[3], d[3], r[4];
  /* -- lookup order ------------------------------------------------------------------ */
  int32_t *sorted_row;    /* [nnz] row of the s-th lookup in (row, position) order; the
                             valid lookups come first, invalid ones hold n0*n1*n2         */
  int32_t *perm;          /* [nnz] original position of the s-th sorted lookup            */
  int32_t *bag_of_sorted; /* [nnz] bag that holds the s-th sorted lookup                  */
  int32_t *slot_of_sorted;/* [nnz] distinct-row slot of the s-th sorted lookup, -1 invalid*/
  int32_t *lookup2row;    /* [nnz] distinct-row slot of original position l, -1 invalid   */
  /* -- distinct rows and prefixes ------------------------------------------------------ */
  int32_t *uniq_row;      /* [U_r] distinct rows, strictly increasing                     */
  int32_t *row_seg;       /* [U_r+1] sorted-lookup range of each distinct row             */
  int32_t *row2pref;      /* [U_r] prefix slot of each distinct row                       */
  int32_t *uniq_pref;     /* [U_p] distinct prefixes i1*n[1]+i2, strictly increasing      */
  int32_t *pref_seg;      /* [U_p+1] distinct-row range of each prefix                    */
  /* -- groupings used by the core-gradient reductions ---------------------------------- */
  int32_t *rows_by_i3;    /* [U_r] distinct-row slots stably sorted by i3                 */
  int32_t *i3_of_sorted;  /* [U_r] the i3 key of rows_by_i3[.] (non-decreasing)           */
  int32_t *i3_seg;        /* [n[2]+1] range in rows_by_i3 of each i3                      */
  int32_t *prefs_by_i2;   /* [U_p] prefix slots stably sorted by i2                       */
  int32_t *i2_seg;        /* [n[1]+1] range in prefs_by_i2 of each i2                     */
  int32_t *i1_seg;        /* [n[0]+1] prefix-slot range of each i1                        */
  int32_t *pref_meta;     /* [max_prefixes][4] per prefix in i2 order: i1, first distinct-row
                             slot, distinct rows, prefix slot (one 16-byte load per prefix for
                             the matrix-core kernels)                                        */
  int32_t *counts;        /* [16] counts[0]=U_r, [1]=U_p, [2]=valid lookups, [3]=nnz,
                             [4]=status bits (1: index out of range, 2: bad offsets)      */
  /* -- float scratch used by forward / backward (contents are transient) --------------- */
  float *rowbuf;          /* [max_rows][D] reconstructed distinct rows                    */
  float *gagg;            /* [max_rows][D] output gradients merged per distinct row       */
  float *hbuf;            /* [max_prefixes][d0*d1*r2] per-prefix right partial gradients;
                             NULL when the table is served by the matrix-core kernels, which
                             keep them on chip                                               */
  float *t3buf;           /* [max_rows][r2*d2] per-row contributions to core 2            */
  float *t1buf;           /* [max_prefixes][d0*r1] per-prefix contributions to core 0     */
  float *partial;         /* segmented-reduction partials                                 */
  float *dg2part;         /* [split][core-1 shape] partial core-1 gradients when the backward
                             workgroups of a table with few core-1 slices are split        */
  void *sort_tmp;         /* radix-sort ping-pong buffers, histograms, scan temporaries   */
  void *prof;             /* HOST, optional tt_prof* attached by the caller (NULL after
                             tt_index_reorder): brackets one kernel with HIP events       */
  void *workspace;        /* the caller's workspace this plan points into                 */
  size_t workspace_bytes;
} tt_plan;

/* Bytes of DEVICE workspace tt_index_reorder needs for this table shape and batch size
 * (0 on invalid arguments).  The workspace must be 256-byte aligned.  The size depends on which
 * kernels serve the table (shape, and whether table->core[1] and core[2] are 16-byte aligned): pass
 * the table with the cores it will be used with.  A backward call whose cores are less aligned than
 * those the workspace was sized for returns TT_ERR_WORKSPACE. */
size_t tt_workspace_bytes(const tt_table *table, int64_t nnz, int64_t num_bags);

/*
 * Index reordering (Section III-G: each batch's lookups are put in increasing
 * index order so that equal TT prefixes become adjacent and reusable; Section
 * III-C: detect which prefix products must be computed; Section III-E: find the
 * distinct rows whose gradients are merged).
 *   indices  DEVICE int64[nnz]        row index of each lookup
 *   offsets  DEVICE int64[num_bags+1] CSR bag offsets
 *   remap    DEVICE int64[num_rows] or NULL: the index bijection f_index of
 *            Section III-G applied before the lookup (row = remap[index]);
 *            NULL = identity.  It changes which row is read.
 *   workspace DEVICE, workspace_bytes >= tt_workspace_bytes(...), 256-byte aligned
 *   plan_out HOST, filled on return (its arrays become valid when the enqueued
 *            work has run).
 * Ties between equal rows keep their original order, so the plan is unique.
 */
tt_status tt_index_reorder(const tt_table *table, const int64_t *indices, const int64_t *offsets,
                           int64_t nnz, int64_t num_bags, const int64_t *remap, void *workspace,
                           size_t workspace_bytes, tt_plan *plan_out, void *stream);

/*
 * Forward (Section III-B): out[b][:] = sum over the lookups l of bag b of the
 * reconstructed row W[index[l]][:], where W[i] = G1[i1] x G2[i2] x G3[i3].
 *   plan != NULL: each distinct prefix product G1[i1] x G2[i2] and each distinct
 *                 row is computed once (batch-level reuse, Section III-C), then
 *                 bags are summed; `indices` may be NULL (the plan holds them).
 *   plan == NULL: naive arm, every lookup runs the full chain (no reuse).
 *   out  DEVICE float[num_bags][D], overwritten.
 * The remap given to tt_index_reorder is baked into the plan; the naive arm
 * reads `indices` as they are.
 */
tt_status tt_emb_bag_forward(const tt_table *table, const tt_plan *plan, const int64_t *indices,
                             const int64_t *offsets, int64_t nnz, int64_t num_bags, float *out,
                             void *stream);

/*
 * Backward (Section III-D backward equation; Section III-E in-advance gradient
 * aggregation): gradients of L w.r.t. the three cores given grad_out[b][:] =
 * dL/d out[b][:].  Gradients of repeated rows add up.
 *   plan != NULL: output gradients are first merged per distinct row, then
 *                 contracted once per distinct row / prefix, and slice gradients
 *                 are combined by sorted segmented reductions.
 *   plan == NULL: naive arm, one contraction per lookup, atomic accumulation.
 *   grad_out DEVICE float[num_bags][D]
 *   dcore    HOST array of 3 DEVICE pointers, core-shaped, fully overwritten
 *            (slices no lookup touches are exactly 0).
 */
tt_status tt_emb_bag_backward(const tt_table *table, const tt_plan *plan, const int64_t *indices,
                              const int64_t *offsets, int64_t nnz, int64_t num_bags,
                              const float *grad_out, float *const dcore[3], void *stream);

/*
 * Gradient-descent update of the cores (training algorithm, update step):
 * G_k <- G_k - lr * dG_k for k = 0,1,2, in place.
 *   plan != NULL: only the slices the batch touched are visited (the others have
 *                 zero gradient, so the result is identical);
 *   plan == NULL: dense sweep over the three cores.
 */
tt_status tt_core_sgd_update(const tt_table *table, const tt_plan *plan,
                             const float *const dcore[3], float lr, void *stream);

/*
 * Backward with the core update fused in (Section III-F, fused TT-core update): the same
 * gradients as tt_emb_bag_backward with a plan, but every gradient slice is applied as
 * G_k <- G_k - lr * dG_k at the point where its reduction completes (the workgroup that holds the
 * finished core-1 strip in registers, the final step of the segmented sums for cores 0 and 2), so
 * no core-shaped gradient is written to or re-read from memory and the separate update launch
 * disappears.  The cores end up bitwise equal to tt_emb_bag_backward followed by
 * tt_core_sgd_update on the same plan; all contractions use the pre-update cores.
 *   plan     required (the naive arm accumulates with atomics and has no completion point);
 *   table->core[k] are updated IN PLACE; no gradient is returned.
 */
tt_status tt_emb_bag_backward_sgd(const tt_table *table, const tt_plan *plan, const int64_t *indices,
                                  const int64_t *offsets, int64_t nnz, int64_t num_bags,
                                  const float *grad_out, float lr, void *stream);

/*
 * Forward by sample-level reuse (Section III-B, reuse equation) on top of the reuse buffer of
 * Section III-C: first the product G1[i1] x G2[i2] of every distinct prefix of the batch is written
 * to `reuse_buffer` (the paper's Reuse Buffer, [prefix slot][(j1,j2)][r2] fp32); then each bag
 * groups its lookups by prefix, sums the core-2 slices G3[:, i3, :] of a group and multiplies the
 * group's buffered product by that sum ONCE -- one second-stage multiplication per (bag, prefix)
 * group instead of one per lookup -- adding the results into the bag's output row.  Same result
 * as tt_emb_bag_forward up to the order of the fp32 additions; bitwise reproducible.
 * It pays when bags are long and their lookups share prefixes; with few lookups per bag the
 * batch-level route of tt_emb_bag_forward (each distinct row once, then a gather) moves less data.
 *   plan          required (built by tt_index_reorder for this batch)
 *   reuse_buffer  DEVICE, 256-byte aligned, at least tt_reuse_buffer_bytes(table, nnz) bytes,
 *                 borrowed until the enqueued work has finished; contents are transient.
 *   out           DEVICE float[num_bags][D], overwritten.
 * tt_reuse_buffer_bytes returns 0 on invalid arguments.
 */
size_t tt_reuse_buffer_bytes(const tt_table *table, int64_t nnz);
tt_status tt_emb_bag_forward_sample(const tt_table *table, const tt_plan *plan, const int64_t *offsets,
                                    int64_t nnz, int64_t num_bags, void *reuse_buffer,
                                    size_t reuse_buffer_bytes, float *out, void *stream);

/*
 * Reduced-precision cores (deployment discussion of the paper: devices with half-precision
 * arithmetic): the three cores are STORED as bf16, all accumulation stays fp32.
 * tt_cores_to_bf16 rounds table->core[0..2] (round to nearest, ties to even) into `bf16_cores`, a
 * DEVICE buffer of tt_bf16_cores_bytes(table) bytes, 256-byte aligned, in a layout private to the
 * library (core 1 is regrouped for the matrix-core kernel).  tt_emb_bag_forward_bf16 is the
 * planned forward of tt_emb_bag_forward reading those copies: the prefix products run on the bf16
 * matrix-core instruction (products of bf16 values are exact in fp32, sums are fp32), the products
 * stay fp32 and the second stage is the fp32 kernel with core-2 values widened exactly.  The result
 * therefore equals the fp32 forward of the ROUNDED cores to fp32 rounding (tolerance 1e-5 as for
 * tt_emb_bag_forward), and differs from the forward of the unrounded cores by at most
 * ((1 + 2^-9)^3 - 1) * sum over the TT paths of |G1 G2 G3|, about 0.6 % of that sum.
 * Only tables the matrix-core kernels serve (d = (4, 8, 4), ranks (32, 32) or (64, 64)):
 * TT_ERR_SHAPE otherwise (0 from the size query).  table->core[] are not read by the forward.
 */
size_t tt_bf16_cores_bytes(const tt_table *table);
tt_status tt_cores_to_bf16(const tt_table *table, void *bf16_cores, size_t bf16_cores_bytes, void *stream);
tt_status tt_emb_bag_forward_bf16(const tt_table *table, const void *bf16_cores, const tt_plan *plan,
                                  const int64_t *offsets, int64_t nnz, int64_t num_bags, float *out,
                                  void *stream);

/*
 * Forward for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  One call = index reorder +
 * planned forward (the result is bitwise that of tt_index_reorder followed by tt_emb_bag_forward
 * with the plan), with the plan's workspace in a static device array of TT_STATIC_SCRATCH_BYTES
 * that the library's code object holds on every GPU it runs on until the process ends.  The call
 * allocates and frees nothing.
 *   indices, offsets, out  DEVICE, as in tt_emb_bag_forward; no remap.
 * Returns TT_ERR_WORKSPACE when the batch needs more than TT_STATIC_SCRATCH_BYTES (at D = 128
 * about 50 000 lookups).  All calls on one GPU share that GPU's array: calls that overlap on one
 * GPU (different streams, or host threads without ordering) race; calls on one stream are safe.
 * Nothing in the array has to be cleared between calls (the reorder initialises what it reads).
 * The first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 * outside a stream capture.  Index errors are skipped silently (there is no plan to query).
 */
#define TT_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
tt_status tt_emb_bag_forward_static(const tt_table *table, const int64_t *indices, const int64_t *offsets,
                                    int64_t nnz, int64_t num_bags, float *out, void *stream);

/*
 * Batched calls: the same four operations for several tables with ONE launch per kernel, so that
 * small tables share the chip with large ones and the host enqueues dozens, not thousands, of
 * launches per step.  All tables of a call must share d[] and r[] (n[] may differ) and must all
 * have a plan or all lack one.  Each item names one table's arguments exactly as in the
 * single-table calls; fields a call does not use are ignored.
 *   items  HOST array of num_tables items (1..256); for reorder, items[t].plan is filled.
 *   desc   DEVICE scratch of at least tt_batch_desc_bytes(num_tables) bytes, 16-byte aligned,
 *          into which the call writes the kernels' per-table descriptors (small launches on
 *          `stream` that carry them as arguments, so the write is ordered like any kernel).  It
 *          is borrowed until the enqueued work has finished: consecutive calls on ONE stream may
 *          share a buffer, calls that may overlap on different streams need different buffers.
 * Results are bitwise identical to the single-table calls.
 * STATUS: switched off.  Every batched call currently returns TT_ERR_UNAVAILABLE without
 * touching the device: the first GPU run of the batched path ended in a memory fault whose cause
 * has not been found yet, so the path stays disabled until it is.  The single-table calls are
 * unaffected (they share the kernels but pass one descriptor by value).
 */
typedef struct {
  const tt_table *table;   /* HOST                                                         */
  tt_plan *plan;           /* HOST; out for reorder, in otherwise (NULL = naive arm)       */
  const int64_t *indices;  /* DEVICE int64[nnz]                                            */
  const int64_t *offsets;  /* DEVICE int64[num_bags+1]                                     */
  int64_t nnz, num_bags;
  const int64_t *remap;    /* DEVICE or NULL (reorder)                                     */
  void *workspace;         /* DEVICE (reorder)                                             */
  size_t workspace_bytes;
  float *out;              /* DEVICE float[num_bags][D] (forward)                          */
  const float *grad_out;   /* DEVICE float[num_bags][D] (backward)                         */
  float *dcore[3];         /* DEVICE core-shaped (backward: written; update: read)         */
} tt_batch_item;

size_t tt_batch_desc_bytes(int num_tables);
tt_status tt_index_reorder_batched(int num_tables, tt_batch_item *items, void *desc,
                                   size_t desc_bytes, void *stream);
tt_status tt_emb_bag_forward_batched(int num_tables, tt_batch_item *items, void *desc,
                                     size_t desc_bytes, void *stream);
tt_status tt_emb_bag_backward_batched(int num_tables, tt_batch_item *items, void *desc,
                                      size_t desc_bytes, void *stream);
tt_status tt_core_sgd_update_batched(int num_tables, tt_batch_item *items, float lr, void *desc,
                                     size_t desc_bytes, void *stream);

/*
 * Fused tables.  TT tables with the same column factors d[] and ranks r[] can be stored as ONE TT
 * table whose core k is the members' cores k laid side by side along the row-factor axis:
 * [r_k][sum over members of n_k][d_k][r_k+1], member t owning the range [o_k(t), o_k(t) + n_k(t)) of
 * that axis (o_k = sum of n_k over the members before t).  Row i = (i1, i2, i3) of member t
 * (index split of Section III-B) is row ((o_1 + i1) * N2 + o_2 + i2) * N3 + o_3 + i3 of the fused
 * table (N_k = sum of n_k): the same three slices, hence the same product (TT-matrix equation,
 * Section II-B), the same bag sums and the same core gradients, found at the members' ranges of the
 * fused cores.  Fused rows that mix slices of different members exist but are never looked up.
 * One reorder, one forward and one backward over the fused table then replace the members' calls:
 * fewer, larger launches (the batched prefix products of Section III-C now batch over tables too).
 *
 * tt_fuse_shape fills fused->num_rows and fused->n[] (d[], r[] and core[] are the caller's):
 * TT_ERR_SHAPE if a row factor sum or the row count does not fit (N1*N2*N3 must stay below 2^31).
 *
 * tt_fuse_lookups maps one batch of every member into the fused table, member after member:
 *   indices, offsets  HOST arrays [num_tables] of DEVICE pointers: member t's int64[nnz[t]] and
 *                     CSR int64[num_bags[t] + 1], as tt_index_reorder takes them
 *   remaps            HOST array of DEVICE pointers or NULL; a non-NULL entry is member t's row
 *                     bijection f_index (int64[num_rows of t]), applied before the split
 *   nnz, num_bags     HOST int64[num_tables]
 *   fused_indices     DEVICE int64[sum nnz]: member t's lookups at [sum of nnz before t, ...);
 *                     an index outside [0, num_rows of t) becomes -1, which tt_index_reorder
 *                     reports and skips like any invalid index
 *   fused_offsets     DEVICE int64[sum num_bags + 1]: member t's bags at [sum of num_bags before
 *                     t, ...), so that rows of `out` / `grad_out` of the fused calls are the
 *                     members' rows, member after member.  An offset outside [0, nnz[t]], a first
 *                     offset other than 0 or a last one other than nnz[t] is written as -1, which
 *                     tt_index_reorder reports as an invalid CSR array.
 * One launch on `stream`; nothing is read on the host.  At most TT_FUSE_MAX_TABLES members.
 */
#define TT_FUSE_MAX_TABLES 32
typedef struct {
  int32_t num_tables;
  int32_t n[TT_FUSE_MAX_TABLES][3];     /* row factors of member t                             */
  int64_t num_rows[TT_FUSE_MAX_TABLES]; /* rows of member t (<= n[t][0]*n[t][1]*n[t][2])       */
} tt_fuse_members;

tt_status tt_fuse_shape(const tt_fuse_members *members, tt_table *fused);
tt_status tt_fuse_lookups(const tt_fuse_members *members, const int64_t *const *indices,
                          const int64_t *const *offsets, const int64_t *const *remaps,
                          const int64_t *nnz, const int64_t *num_bags, int64_t *fused_indices,
                          int64_t *fused_offsets, void *stream);

/*
 * Index-graph edges of one batch (Section III-G, index-graph generation algorithm): the weighted
 * co-occurrence graph the offline index bijection is built from.  Offline preprocessing, not part
 * of a training step.
 *   node of a lookup = max(rank[index], hot_thresh) - hot_thresh, with rank[] the frequency rank
 *   of every row (0 = most frequent); node 0 (all hot rows) is dropped.  Every bag contributes one
 *   pair (u < v) per two of its distinct nodes; a bag with more than max_group (<= 64) distinct
 *   nodes keeps its max_group smallest ones, and only the first 256 lookups of a bag are looked at.
 *   Equal pairs are merged; weight = number of bags that hold both ends.
 *   indices, offsets  DEVICE, as in tt_index_reorder (invalid indices are skipped)
 *   rank              DEVICE int32[num_rows]
 *   workspace         DEVICE, 256-byte aligned, tt_index_graph_workspace_bytes(num_bags, max_pairs)
 *   edge_u/v/w        DEVICE int32[max_pairs] each: the edges, sorted by (u, v), weights in edge_w
 *   counts            DEVICE int32[4]: [0] pairs before merging, [1] edges, [2] 1 if the batch has
 *                     more than max_pairs pairs (then no edge is produced)
 * The result is unique (integer work, stable sorts).
 */
size_t tt_index_graph_workspace_bytes(int64_t num_bags, int64_t max_pairs);
tt_status tt_index_graph_edges(const int64_t *indices, const int64_t *offsets, int64_t nnz, int64_t num_bags,
                               const int32_t *rank, int64_t num_rows, int64_t hot_thresh, int32_t max_group,
                               void *workspace, size_t workspace_bytes, int64_t max_pairs, int32_t *edge_u,
                               int32_t *edge_v, int32_t *edge_w, int32_t *counts, void *stream);

/*
 * Waits for `stream`, copies the plan's device-side counters to the host and
 * reports deferred errors.  counts_out (HOST, nullable) receives
 * {U_r, U_p, valid lookups, status bits}.  Returns TT_ERR_INDEX_RANGE if any
 * index was out of range or the offsets were not a valid CSR array.
 */
tt_status tt_plan_status(const tt_plan *plan, void *stream, int64_t counts_out[4]);

const char *tt_strerror(tt_status status);

/*
 * Kernel timing helper for benchmarks (not needed by the operator itself, and the one place
 * where the library owns anything: a host object holding HIP events).  A tt_prof selects one
 * kernel of the planned path; while it is attached to a plan (plan->prof), every launch of that
 * kernel made with the plan is bracketed by two HIP events recorded on the launch stream.
 * tt_prof_collect waits for the recorded events, returns the summed duration and the number of
 * launches since the last collect, and rearms the object.  At most `capacity` launches are
 * recorded between two collects; later ones run untimed.
 */
typedef enum {
  TT_KERNEL_FWD_CONTRACT = 0, /* prefix products + distinct rows (forward)                   */
  TT_KERNEL_BAG_SUM = 1,      /* per-bag sum of distinct rows                                */
  TT_KERNEL_GRAD_MERGE = 2,   /* stage 1 of merging grad_out per distinct row                */
  TT_KERNEL_BWD_CONTRACT = 3, /* backward contraction kernel (without the sum of split parts)  */
  TT_KERNEL_SORT_SCATTER = 4, /* one radix-sort scatter pass of the main lookup sort         */
  TT_KERNEL_SGD = 5,          /* core update                                                 */
  TT_KERNEL_P12_FILL = 6,     /* reuse buffer of the sample-level forward                    */
  TT_KERNEL_BAG_CHAINS = 7,   /* per-bag chains of the sample-level forward                  */
  TT_KERNEL_COUNT = 8
} tt_kernel;

typedef struct tt_prof tt_prof;
tt_prof *tt_prof_create(int kernel, int capacity); /* NULL on failure                        */
void tt_prof_destroy(tt_prof *prof);
/* HOST out-params; returns TT_ERR_HIP if an event query fails */
tt_status tt_prof_collect(tt_prof *prof, double *total_ms, int64_t *launches);
const char *tt_kernel_name(int kernel);

#ifdef __cplusplus
}
#endif
#endif /* TT_EMB_H_ */
