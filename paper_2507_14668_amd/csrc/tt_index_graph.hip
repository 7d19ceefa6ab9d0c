// Index-graph edges on the GPU (paper Section III-G, index-graph generation algorithm): the
// co-occurrence graph from which the offline index bijection is built.  For one batch,
//   node(l) = max(rank[index[l]], hot) - hot      frequency rank shifted by the hot threshold
//                                                  (all hot rows collapse to node 0, which is dropped)
//   every bag contributes one edge per pair of its distinct nodes (bags with more than max_group
//   distinct nodes keep their max_group smallest, i.e. most frequent, ones)
//   equal pairs are merged: weight = number of bags that hold both ends.
// Steps: pairs per bag -> exclusive scan -> pair list -> stable LSD radix sort by v, then by u
// (the sort kernels of the reorder plan) -> run heads -> (u, v, w), u < v, sorted by (u, v).
// All integer work; the result is unique.
#include <string.h>

#include "tt_internal.h"

#define TT_EDGE_BAG_CAP 256  // lookups of a bag that are looked at (four wavefront rounds)
#define TT_EDGE_MAX_GROUP 64

namespace {

struct EdgeArgs {
  const int64_t *indices, *offsets;
  const int32_t *rank;
  long long num_rows, hot, nnz;
  int num_bags, max_group;
  long long cap;          // pair capacity
  int32_t *bag_off;       // [num_bags + 1] pair offset of each bag
  int32_t *counts;        // [0] pairs, [1] edges, [2] status (1: more pairs than capacity)
  int32_t *pair_v, *pair_u;  // first sort: key = v, payload = u
};

// The bag's distinct non-hot nodes in increasing order, at most max_group of them, in `sorted`
// (LDS, this wavefront's, TT_EDGE_MAX_GROUP ints); returns their number.  `nodes` and `uniq` are this
// wavefront's LDS scratch of TT_EDGE_BAG_CAP ints each.  Executed by all lanes of the wavefront.
__device__ int bag_nodes(const EdgeArgs &a, int bag, int *nodes, int *uniq, int *sorted) {
  const int lane = threadIdx.x & (TT_WAVE - 1);
  // offsets are clamped to [0, nnz] so that a malformed CSR array cannot index out of bounds
  const long long o0 = a.offsets[bag], o1 = a.offsets[bag + 1];
  const long long lo = o0 < 0 ? 0 : (o0 > a.nnz ? a.nnz : o0), hi = o1 < lo ? lo : (o1 > a.nnz ? a.nnz : o1);
  const int len = (int)((hi - lo) < TT_EDGE_BAG_CAP ? (hi - lo) : TT_EDGE_BAG_CAP);
  for (int p = lane; p < len; p += TT_WAVE) {
    const long long row = a.indices[lo + p];
    int node = 0;
    if (row >= 0 && row < a.num_rows) {
      const long long r = a.rank[row];
      node = r > a.hot ? (int)(r - a.hot) : 0;
    }
    nodes[p] = node;
  }
  tt_wave_lds_order();
  // uniq[p] = the node at its first occurrence, 0 elsewhere (and for hot rows and invalid lookups)
  int kept = 0;
  for (int p0 = 0; p0 < len; p0 += TT_WAVE) {  // uniform trip count
    const int p = p0 + lane;
    const int x = p < len ? nodes[p] : 0;
    bool first = x > 0;
    for (int q = 0; q < p && first; ++q) first = nodes[q] != x;
    if (p < len) uniq[p] = first ? x : 0;
    kept += __popcll(__ballot(first));
  }
  tt_wave_lds_order();
  // position of each distinct node = number of smaller distinct nodes
  for (int p = lane; p < len; p += TT_WAVE) {
    const int x = uniq[p];
    if (x > 0) {
      int pos = 0;
      for (int q = 0; q < len; ++q) {
        const int y = uniq[q];
        pos += (y > 0 && y < x) ? 1 : 0;
      }
      if (pos < a.max_group) sorted[pos] = x;
    }
  }
  tt_wave_lds_order();
  return kept < a.max_group ? kept : a.max_group;
}

__global__ void __launch_bounds__(TT_BLOCK)
k_edge_count(EdgeArgs a) {
  __shared__ int s_nodes[TT_BLOCK / TT_WAVE][TT_EDGE_BAG_CAP], s_uniq[TT_BLOCK / TT_WAVE][TT_EDGE_BAG_CAP];
  __shared__ int s_sorted[TT_BLOCK / TT_WAVE][TT_EDGE_MAX_GROUP];
  const int wave = threadIdx.x / TT_WAVE, lane = threadIdx.x & (TT_WAVE - 1);
  const int bag = blockIdx.x * (TT_BLOCK / TT_WAVE) + wave;
  if (bag >= a.num_bags) return;  // uniform for the wavefront; no workgroup barrier in this kernel
  const int m = bag_nodes(a, bag, s_nodes[wave], s_uniq[wave], s_sorted[wave]);
  if (lane == 0) a.bag_off[bag] = m * (m - 1) / 2;
}

// One workgroup: exclusive scan of the per-bag pair counts in place; total and status.
__global__ void __launch_bounds__(TT_BLOCK)
k_edge_scan_bags(EdgeArgs a) {
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  long long carry = 0;
  for (int base = 0; base < a.num_bags; base += TT_BLOCK) {
    const int b = base + threadIdx.x;
    const int v = b < a.num_bags ? a.bag_off[b] : 0;
    int total;
    const int ex = tt_block_excl_scan(v, tmp, &total);
    // offsets are only used when the total fits the capacity (< 2^31), so the narrowing is safe then
    if (b < a.num_bags) a.bag_off[b] = (int)(carry + ex);
    carry += total;
  }
  if (threadIdx.x == 0) {
    const bool fits = carry <= a.cap;
    a.bag_off[a.num_bags] = fits ? (int)carry : 0;
    a.counts[0] = fits ? (int)carry : 0;
    a.counts[1] = 0;
    a.counts[2] = fits ? 0 : 1;
  }
}

__global__ void __launch_bounds__(TT_BLOCK)
k_edge_pairs(EdgeArgs a) {
  __shared__ int s_nodes[TT_BLOCK / TT_WAVE][TT_EDGE_BAG_CAP], s_uniq[TT_BLOCK / TT_WAVE][TT_EDGE_BAG_CAP];
  __shared__ int s_sorted[TT_BLOCK / TT_WAVE][TT_EDGE_MAX_GROUP];
  const int wave = threadIdx.x / TT_WAVE, lane = threadIdx.x & (TT_WAVE - 1);
  const int bag = blockIdx.x * (TT_BLOCK / TT_WAVE) + wave;
  if (bag >= a.num_bags) return;  // uniform for the wavefront
  if (a.counts[2] != 0) return;   // more pairs than capacity: nothing is written
  const int m = bag_nodes(a, bag, s_nodes[wave], s_uniq[wave], s_sorted[wave]);
  const int base = a.bag_off[bag];
  const int *sorted = s_sorted[wave];
  for (int i = 0; i + 1 < m; ++i) {
    const int row0 = base + i * (m - 1) - i * (i - 1) / 2;  // pairs (i, i+1 .. m-1) start here
    for (int j = i + 1 + lane; j < m; j += TT_WAVE) {
      a.pair_u[row0 + (j - i - 1)] = sorted[i];
      a.pair_v[row0 + (j - i - 1)] = sorted[j];
    }
  }
}

// ---- run heads of the sorted pair list -> edges -------------------------------------------------
struct EmitArgs {
  const int32_t *u, *v;     // sorted by (u, v)
  const int32_t *counts;    // [0] pairs
  int32_t *counts_out;      // [1] edges
  int32_t *tile_sums;       // [tiles]
  int32_t *edge_start;      // [cap + 1]
  int32_t *eu, *ev, *ew;
  int tiles;
};

__device__ __forceinline__ int pair_head(const EmitArgs &a, int s, int n) {
  if (s >= n) return 0;
  return s == 0 || a.u[s] != a.u[s - 1] || a.v[s] != a.v[s - 1];
}

__global__ void __launch_bounds__(TT_BLOCK)
k_edge_heads(EmitArgs a) {
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  const int n = a.counts[0];
  int h = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) h += pair_head(a, (blockIdx.x * TT_BLOCK + threadIdx.x) * 4 + i, n);
  int total;
  (void)tt_block_excl_scan(h, tmp, &total);
  if (threadIdx.x == 0) a.tile_sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(TT_BLOCK)
k_edge_scan_tiles(EmitArgs a) {
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int carry = 0;
  for (int base = 0; base < a.tiles; base += TT_BLOCK) {
    const int t = base + threadIdx.x;
    const int v = t < a.tiles ? a.tile_sums[t] : 0;
    int total;
    const int ex = tt_block_excl_scan(v, tmp, &total);
    if (t < a.tiles) a.tile_sums[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    a.counts_out[1] = carry;
    a.edge_start[carry] = a.counts[0];
  }
}

__global__ void __launch_bounds__(TT_BLOCK)
k_edge_emit(EmitArgs a) {
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  const int n = a.counts[0];
  const int s0 = (blockIdx.x * TT_BLOCK + threadIdx.x) * 4;
  int hd[4], h = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) { hd[i] = pair_head(a, s0 + i, n); h += hd[i]; }
  int total;
  int pos = a.tile_sums[blockIdx.x] + tt_block_excl_scan(h, tmp, &total);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (hd[i]) {
      a.eu[pos] = a.u[s0 + i];
      a.ev[pos] = a.v[s0 + i];
      a.edge_start[pos] = s0 + i;
      ++pos;
    }
}

__global__ void __launch_bounds__(TT_BLOCK)
k_edge_weights(EmitArgs a) {
  const int e = blockIdx.x * TT_BLOCK + threadIdx.x;
  if (e < a.counts_out[1]) a.ew[e] = a.edge_start[e + 1] - a.edge_start[e];
}

size_t pad64(size_t ints) { return (ints + 63) & ~(size_t)63; }

struct EdgeLayout {
  size_t bag_off, counts, ka, va, kb, vb, hist, bin_total, tile_sums, edge_start, total;
};

EdgeLayout edge_layout(long long num_bags, long long cap) {
  EdgeLayout L;
  size_t at = 0;
  auto take = [&](size_t ints) { const size_t o = at; at += pad64(ints); return o; };
  const size_t tiles = (size_t)tt_ceil_div(cap, TT_SORT_TILE) + 1;
  L.bag_off = take((size_t)num_bags + 1);
  L.counts = take(16);
  L.ka = take((size_t)cap); L.va = take((size_t)cap); L.kb = take((size_t)cap); L.vb = take((size_t)cap);
  L.hist = take(tiles << TT_SORT_MAX_BITS);
  L.bin_total = take((size_t)1 << TT_SORT_MAX_BITS);
  L.tile_sums = take(tiles);
  L.edge_start = take((size_t)cap + 1);
  L.total = at * sizeof(int32_t);
  return L;
}

}  // namespace

size_t ttk_index_graph_workspace_bytes(long long num_bags, long long max_pairs) {
  return edge_layout(num_bags, max_pairs).total;
}

tt_status ttk_index_graph_edges(const int64_t *indices, const int64_t *offsets, long long nnz, long long num_bags,
                                const int32_t *rank, long long num_rows, long long hot, int max_group,
                                void *workspace, long long max_pairs, int32_t *eu, int32_t *ev, int32_t *ew,
                                int32_t *counts_out, hipStream_t s) {
  const EdgeLayout L = edge_layout(num_bags, max_pairs);
  int32_t *w = (int32_t *)workspace;
  int key_bits = 1;
  while (((long long)1 << key_bits) < num_rows) ++key_bits;  // node ids are below num_rows
  const int passes = ttk_radix_passes(key_bits);  // both sorts have the same key width
  // The sort leaves its result in the (a) buffers and wants its input in (a) for an even number of
  // passes, in (b) for an odd one.  Sort 1: key = v, payload = u.  Sort 2: key = u, payload = v, on
  // the result of sort 1 with the roles of the arrays exchanged.
  int32_t *ka = w + L.ka, *va = w + L.va, *kb = w + L.kb, *vb = w + L.vb;
  const bool in_a = (passes % 2) == 0;
  EdgeArgs ea;
  ea.indices = indices; ea.offsets = offsets; ea.rank = rank;
  ea.num_rows = num_rows; ea.hot = hot; ea.nnz = nnz;
  ea.num_bags = (int)num_bags; ea.max_group = max_group;
  ea.cap = max_pairs;
  ea.bag_off = w + L.bag_off;
  ea.counts = counts_out;
  ea.pair_v = in_a ? ka : kb;
  ea.pair_u = in_a ? va : vb;
  const int wpb = TT_BLOCK / TT_WAVE;
  const int bag_grid = num_bags > 0 ? tt_ceil_div(num_bags, wpb) : 1;
  hipLaunchKernelGGL(k_edge_count, dim3(bag_grid), dim3(TT_BLOCK), 0, s, ea);
  hipLaunchKernelGGL(k_edge_scan_bags, dim3(1), dim3(TT_BLOCK), 0, s, ea);
  hipLaunchKernelGGL(k_edge_pairs, dim3(bag_grid), dim3(TT_BLOCK), 0, s, ea);
  if (tt_launch_status() != TT_OK) return TT_ERR_HIP;

  // sort 1 result: (ka: v, va: u).  Sort 2 input (key = u, payload = v) = (va, ka).
  TTDev d;
  memset(&d, 0, sizeof(d));
  d.plan.counts = counts_out;
  d.plan.max_rows = max_pairs;
  d.tmp.hist = w + L.hist;
  d.tmp.bin_total = w + L.bin_total;
  d.plan.i3_of_sorted = ka; d.plan.rows_by_i3 = va; d.tmp.k3_alt = kb; d.tmp.v3_alt = vb;
  tt_status st = ttk_sort_slot1(d, key_bits, s);
  if (st != TT_OK) return st;
  int32_t *u_sorted, *v_sorted;
  if (in_a) {  // input of sort 2 must sit in its (a) buffers: a' = (va, ka), b' = (vb, kb); result in a'
    d.plan.i3_of_sorted = va; d.plan.rows_by_i3 = ka; d.tmp.k3_alt = vb; d.tmp.v3_alt = kb;
    u_sorted = va; v_sorted = ka;
  } else {     // input must sit in (b'): b' = (va, ka), a' = (vb, kb); result in a'
    d.plan.i3_of_sorted = vb; d.plan.rows_by_i3 = kb; d.tmp.k3_alt = va; d.tmp.v3_alt = ka;
    u_sorted = vb; v_sorted = kb;
  }
  st = ttk_sort_slot1(d, key_bits, s);
  if (st != TT_OK) return st;

  EmitArgs em;
  em.u = u_sorted; em.v = v_sorted;
  em.counts = counts_out; em.counts_out = counts_out;
  em.tile_sums = w + L.tile_sums;
  em.edge_start = w + L.edge_start;
  em.eu = eu; em.ev = ev; em.ew = ew;
  em.tiles = tt_ceil_div(max_pairs, TT_SORT_TILE) > 0 ? tt_ceil_div(max_pairs, TT_SORT_TILE) : 1;
  hipLaunchKernelGGL(k_edge_heads, dim3(em.tiles), dim3(TT_BLOCK), 0, s, em);
  hipLaunchKernelGGL(k_edge_scan_tiles, dim3(1), dim3(TT_BLOCK), 0, s, em);
  hipLaunchKernelGGL(k_edge_emit, dim3(em.tiles), dim3(TT_BLOCK), 0, s, em);
  hipLaunchKernelGGL(k_edge_weights, dim3(em.tiles * 4), dim3(TT_BLOCK), 0, s, em);
  return tt_launch_status();
}
