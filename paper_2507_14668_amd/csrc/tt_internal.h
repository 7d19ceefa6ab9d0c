// Internal declarations shared by the HIP translation units of the TT embedding-bag library.
// Nothing here is part of the C ABI (see include/tt_emb.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "tt_emb.h"

// Derived shape of one table, passed by value to kernels.
struct TTShape {
  int n1, n2, n3;
  int d1, d2, d3;
  int R1, R2;
  int D;    // d1*d2*d3   columns of a row
  int S1;   // d1*R1      floats of a core-0 slice
  int S2;   // d2*R2      floats of one r1-chunk of a core-1 slice
  int S3;   // R2*d3      floats of a core-2 slice
  int P;    // d1*d2*R2   floats of a prefix product G1[i1] x G2[i2]
  int R2p;  // padded LDS row stride for [.][R2] tiles (odd, avoids bank conflicts)
  int sentinel;       // n1*n2*n3, sort key of an invalid lookup
  // exact division of a non-negative int by n3 / n2 without a divide: q = (x * mul) >> (31 + sh)
  // with mul = ceil(2^(31+sh) / n), sh = bit length of n - 1 (valid for every x < 2^31)
  unsigned mul3, sh3, mul2, sh2;
  long long num_rows;
};

#define TT_WAVE 64
#define TT_BLOCK 256

// ---- radix sort geometry ----------------------------------------------------------------
#ifndef TT_SORT_ITEMS
#define TT_SORT_ITEMS 4
#endif
#define TT_SORT_TILE (TT_BLOCK * TT_SORT_ITEMS)  // keys per workgroup per pass
#define TT_SORT_MAX_BITS 10                      // digit width limit (1024 bins)

// ---- matrix-core kernels -------------------------------------------------------------------
#define TT_MP 8  // distinct prefixes per chunk: two 16-row MFMA tiles of (prefix, j1) rows

// ---- segmented-reduction geometry -----------------------------------------------------------
#ifndef TT_SEG_MIN_CHUNK
#define TT_SEG_MIN_CHUNK 8   // smallest stage-1 chunk of the two-stage segmented sum (sizes the partials)
#endif
#define TT_SEG_MAX_CHUNK 64
#ifndef TT_SEG_UNROLL
#define TT_SEG_UNROLL 4      // gathers a lane group keeps in flight (8 and 16 measured slower: fewer resident lane groups)
#endif

static inline int tt_ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

static inline void tt_div_constants(int n, unsigned *mul, unsigned *sh) {
  unsigned l = 0;
  while ((1ll << l) < n) ++l;  // bit length of n - 1
  *sh = l;
  *mul = (unsigned)((((unsigned long long)1 << (31 + l)) + (unsigned long long)n - 1) / (unsigned long long)n);
}

// Sort scratch carved from plan->sort_tmp (all int32 arrays).
struct TTSortTmp {
  int32_t *keys_alt, *vals_alt;    // [nnz] ping-pong partner of (sorted_row, perm)
  int32_t *bag_tmp;                // [nnz] bag of each original lookup position
  int32_t *k3_alt, *v3_alt;        // [max_rows]
  int32_t *k2, *k2_alt, *v2_alt;   // [max_prefixes]
  int32_t *hist;                   // [bins][tiles] per-tile digit histograms
  int32_t *bin_total;              // [bins]
  int32_t *tile_sums;              // [2][tiles] head counts per tile of the unique pass
};
TTSortTmp tt_sort_tmp_view(const tt_plan *plan);
size_t tt_sort_tmp_bytes(int64_t nnz, int64_t max_rows, int64_t max_prefixes);

// Everything a kernel needs to know about one table of a call.  A single-table call passes one
// TTDev by value as a kernel argument; a batched call uploads an array of them and the kernels
// pick theirs with blockIdx.y, so that one launch serves every table of the batch.
struct TTDev {
  TTShape sh;
  const float *g[3];       // cores
  float *dg[3];            // core gradients (backward / update)
  tt_plan plan;            // device pointers of the plan (host-only fields unused on the device)
  TTSortTmp tmp;           // sort scratch of the plan
  const int64_t *indices, *offsets, *remap;
  const float *grad_out;
  float *out;
  float *p12buf;           // reuse buffer [prefix slot][(j1,j2)][r2] of the sample-level forward
  int nnz, num_bags;
  int sort_tiles;          // radix tiles of the main lookup sort (hist row length)
  int strips;              // contributions per prefix in t1buf: one per strip of the core-1 slice (matrix-core path), else 1
  float lr;
  int fused;               // backward applies G <- G - lr*dG where each gradient slice is completed
  int mfma;                // served by the matrix-core kernels (shape supported, operands aligned)
  int bwd_split;           // workgroups that share one (i2, strip) of the backward matrix-core kernel
};

struct TTBatch {
  int T;              // tables in the call
  const TTDev *host;  // [T] host copies (grid sizing)
  const TTDev *dev;   // [T] device copies, or nullptr: single table passed by value
};

// Streaming accesses (non-temporal): data that a launch writes and no kernel of the path reads again
// (bag sums), or reads exactly once (the output gradients of one-lookup bags, per-row hand-off
// buffers), should not displace the rows and slices that are gathered many times from the caches.
// Measured at config 5 (fused tables): gradient merge 103 -> 86 us.  Output gradients of multi-lookup
// bags are gathered once per lookup and must stay cached (config 4: 49 -> 62 us if streamed).
#ifdef __HIPCC__
typedef float tt_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void tt_store_stream4(float *dst, float a, float b, float c, float d) {
  tt_f32x4 v = {a, b, c, d};
  __builtin_nontemporal_store(v, reinterpret_cast<tt_f32x4 *>(dst));
}
__device__ __forceinline__ float4 tt_load_stream4(const float *src) {
  const tt_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const tt_f32x4 *>(src));
  return make_float4(v.x, v.y, v.z, v.w);
}
#endif

template <bool BATCHED> struct TTArg;
template <> struct TTArg<false> {
  TTDev one;
#ifdef __HIPCC__
  __device__ __forceinline__ const TTDev &get() const { return one; }
#endif
};
template <> struct TTArg<true> {
  const TTDev *arr;
#ifdef __HIPCC__
  __device__ __forceinline__ const TTDev &get() const { return arr[blockIdx.y]; }
#endif
};

// K is a kernel template whose first template parameter is `bool BATCHED` and whose first
// argument is TTArg<BATCHED>; TARGS are its remaining template arguments (may be empty).
#define TT_LAUNCH(K, gx, bs, lds, s, batch, ...)                                                  \
  do {                                                                                            \
    if ((batch).dev)                                                                              \
      hipLaunchKernelGGL((K<true>), dim3((unsigned)(gx), (unsigned)(batch).T), dim3(bs), lds, s,  \
                         TTArg<true>{(batch).dev}, ##__VA_ARGS__);                                \
    else                                                                                          \
      hipLaunchKernelGGL((K<false>), dim3((unsigned)(gx)), dim3(bs), lds, s,                      \
                         TTArg<false>{(batch).host[0]}, ##__VA_ARGS__);                           \
  } while (0)
#define TT_LAUNCH_T(K, TARGS, gx, bs, lds, s, batch, ...)                                         \
  do {                                                                                            \
    if ((batch).dev)                                                                              \
      hipLaunchKernelGGL((K<true, TARGS>), dim3((unsigned)(gx), (unsigned)(batch).T), dim3(bs),   \
                         lds, s, TTArg<true>{(batch).dev}, ##__VA_ARGS__);                        \
    else                                                                                          \
      hipLaunchKernelGGL((K<false, TARGS>), dim3((unsigned)(gx)), dim3(bs), lds, s,               \
                         TTArg<false>{(batch).host[0]}, ##__VA_ARGS__);                           \
  } while (0)

// Launchers (host).  Each enqueues kernels on `s` for every table of the batch and returns the
// launch status.  All tables of a batch share d[] and r[] (checked by the caller).
tt_status ttk_reorder(const TTBatch &b, hipStream_t s);
// The stable LSD radix sort of the plan on caller-chosen buffers: sorts the (key, payload) pairs of
// sort slot 1 -- (plan.i3_of_sorted, plan.rows_by_i3) with partners (tmp.k3_alt, tmp.v3_alt), count in
// plan.counts[0], capacity plan.max_rows, scratch tmp.hist / tmp.bin_total -- by keys of key_bits bits.
// Input in the first pair for an even number of passes, in the partners for an odd one; result in the
// first pair.
int ttk_radix_passes(int key_bits);
tt_status ttk_sort_slot1(const TTDev &d, int key_bits, hipStream_t s);
size_t ttk_index_graph_workspace_bytes(long long num_bags, long long max_pairs);
// Fused tables: sums of the members' row factors (with the limits of a table), and the one-launch
// map of the members' lookups and bag offsets into the fused table.
tt_status ttk_fuse_shape(const tt_fuse_members *members, long long N[3]);
tt_status ttk_fuse_lookups(const tt_fuse_members *members, const int64_t *const *indices,
                           const int64_t *const *offsets, const int64_t *const *remaps,
                           const int64_t *nnz, const int64_t *num_bags, int64_t *fused_indices,
                           int64_t *fused_offsets, hipStream_t s);
tt_status ttk_index_graph_edges(const int64_t *indices, const int64_t *offsets, long long nnz, long long num_bags,
                                const int32_t *rank, long long num_rows, long long hot, int max_group,
                                void *workspace, long long max_pairs, int32_t *eu, int32_t *ev, int32_t *ew,
                                int32_t *counts_out, hipStream_t s);
tt_status ttk_forward_plan(const TTBatch &b, hipStream_t s);
bool ttk_forward_mfma_supported(const TTShape &sh);
tt_status ttk_forward_mfma(const TTBatch &b, hipStream_t s);
// number of strips (16 values of r2, all j2) a core-1 slice is cut into by the backward matrix-core
// kernel (1 when the shape is served by the plain-ALU kernels); t1buf holds one contribution per strip
int ttk_mfma_strips(const TTShape &sh);
// The backward matrix-core kernel has n2 * strips workgroups, two per compute unit; a table with few
// core-1 slices leaves most of the 256 CUs idle, so the chunks of one (i2, strip) are then dealt to `split`
// workgroups that write partial core-1 gradients, summed in a fixed order by a second kernel.
int ttk_bwd_split(const TTShape &sh);
#define TT_BWD_MAX_SPLIT 8
tt_status ttk_backward_mfma(const TTBatch &b, hipStream_t s);
// the matrix-core kernels serve a table when they support its shape and cores 1 and 2 are 16-byte
// aligned (they read core-1 rows and core-2 slices as float4)
static inline bool ttk_mfma_selected(const TTShape &sh, const float *core1, const float *core2) {
  return ttk_forward_mfma_supported(sh) && ((uintptr_t)core1 % 16) == 0 && ((uintptr_t)core2 % 16) == 0;
}
// a batch takes the matrix-core kernels only if every table of it does
static inline bool ttk_batch_mfma(const TTBatch &b) {
  for (int t = 0; t < b.T; ++t)
    if (!b.host[t].mfma) return false;
  return true;
}
// sample-level reuse forward: reuse buffer of prefix products, then one chain per (bag, prefix) group
tt_status ttk_forward_sample(const TTBatch &b, hipStream_t s);
// the matrix-core forward kernel with its second stage replaced by a store of the prefix products
tt_status ttk_forward_mfma_p12(const TTBatch &b, hipStream_t s);
// the matrix-core forward kernel on bf16 copies of the cores (d.g[k] then point at bf16 data)
tt_status ttk_forward_mfma_bf16(const TTBatch &b, hipStream_t s);
tt_status ttk_bag_sum(const TTBatch &b, hipStream_t s);
// byte offsets of the three bf16 cores inside the buffer tt_cores_to_bf16 fills, and its size
void ttk_bf16_layout(const TTShape &sh, size_t off[3], size_t *total);
tt_status ttk_cores_to_bf16(const TTShape &sh, const float *const core[3], void *buf, hipStream_t s);
tt_status ttk_forward_naive(const TTBatch &b, hipStream_t s);
tt_status ttk_backward_plan(const TTBatch &b, hipStream_t s);
tt_status ttk_backward_naive(const TTBatch &b, hipStream_t s);
tt_status ttk_sgd(const TTBatch &b, bool touched_only, hipStream_t s);

template <class F> static inline long long tt_batch_max(const TTBatch &b, F f) {
  long long m = 0;
  for (int t = 0; t < b.T; ++t) {
    const long long v = f(b.host[t]);
    if (v > m) m = v;
  }
  return m;
}

// Brackets the launches made inside its scope with HIP events when the plan carries a tt_prof
// that selects `kernel`.
struct tt_prof {
  int kernel;
  int capacity;
  int used;
  hipEvent_t *ev;  // [2 * capacity]: start, stop
};
struct TTProfScope {
  tt_prof *p;
  hipStream_t s;
  bool record;
  // record = false: the scope only hands out the event pair (start(), stop()) for ONE launch made with
  // hipExtLaunchKernelGGL, which stamps them with that kernel's own begin and end -- the duration a
  // kernel trace reports, without the dispatch gap an event recorded in front of the launch includes.
  TTProfScope(const tt_plan *plan, int kernel, hipStream_t stream, bool record_events = true)
      : p(nullptr), s(stream), record(record_events) {
    tt_prof *q = plan ? (tt_prof *)plan->prof : nullptr;
    if (q && q->kernel == kernel && q->used < q->capacity) {
      p = q;
      if (record) (void)hipEventRecord(p->ev[2 * p->used], s);
    }
  }
  hipEvent_t start() const { return p ? p->ev[2 * p->used] : nullptr; }
  hipEvent_t stop() const { return p ? p->ev[2 * p->used + 1] : nullptr; }
  ~TTProfScope() {
    if (p) {
      if (record) (void)hipEventRecord(p->ev[2 * p->used + 1], s);
      ++p->used;
    }
  }
};

static inline tt_status tt_launch_status() {
  return hipGetLastError() == hipSuccess ? TT_OK : TT_ERR_HIP;
}

// ---- device helpers -----------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ int tt_div(int x, unsigned mul, unsigned sh) {
  return (int)(((unsigned long long)(unsigned)x * mul) >> (31 + sh));
}
// Orders the LDS accesses of the lanes of one wavefront (a wavefront executes them in program
// order; this keeps the compiler from moving them across).
__device__ __forceinline__ void tt_wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ int tt_wave_incl_scan(int v) {
  const int lane = threadIdx.x & (TT_WAVE - 1);
#pragma unroll
  for (int o = 1; o < TT_WAVE; o <<= 1) {
    int t = __shfl_up(v, o, TT_WAVE);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive scan of one int per thread over a TT_BLOCK-thread workgroup.
// `tmp` is LDS with at least TT_BLOCK/TT_WAVE + 1 ints.  Returns the exclusive prefix;
// *total receives the workgroup sum.  Contains two barriers.
__device__ __forceinline__ int tt_block_excl_scan(int v, int *tmp, int *total) {
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;
  int incl = tt_wave_incl_scan(v);
  if (lane == TT_WAVE - 1) tmp[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < TT_BLOCK / TT_WAVE; ++w) {
    int x = tmp[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  *total = tot;
  return base + incl - v;
}

__device__ __forceinline__ float tt_wave_sum(float v) {
#pragma unroll
  for (int o = TT_WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, TT_WAVE);
  return v;
}
#endif
