// Index reordering for the TT embedding bag (paper Sections III-C, III-E, III-G).
//
// The paper elects one thread per (i1,i2) prefix with an atomic compare-and-swap
// on a flag array and hands out reuse-buffer slots with an atomic counter.  Here
// the same information -- which prefix products and which rows are distinct --
// comes from a stable LSD radix sort of the lookups by row followed by a
// head-flag scan, so slots are the ranks in sorted order (deterministic), no
// flag array of size N/n3 is needed, and equal rows / prefixes are contiguous
// for the segmented reductions of the backward pass.
//
// All counts stay on the device: later kernels read U_r / U_p from plan->counts.
#include "tt_internal.h"

namespace {

// ------------------------------------------------------------------ key extraction
template <bool BATCHED>
__global__ void k_init_counts(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  if (threadIdx.x < 16) d.plan.counts[threadIdx.x] = (threadIdx.x == 3) ? d.nnz : 0;
  // a table without lookups has no workgroup that would write the terminal segment entries
  if (threadIdx.x == 16) d.plan.row_seg[0] = 0;
  if (threadIdx.x == 17) d.plan.pref_seg[0] = 0;
}

// One thread per lookup: validate, apply the optional bijection, emit (row, position) and the
// bag holding the position.  Threads b <= num_bags also validate the CSR offsets.
template <bool BATCHED>
__global__ void k_extract_keys(TTArg<BATCHED> a, int in_a) {
  const TTDev &d = a.get();
  const int64_t *__restrict__ indices = d.indices, *__restrict__ offsets = d.offsets,
                *__restrict__ remap = d.remap;
  const int nnz = d.nnz, num_bags = d.num_bags, sentinel = d.sh.sentinel;
  const long long num_rows = d.sh.num_rows;
  int32_t *__restrict__ keys = in_a ? d.plan.sorted_row : d.tmp.keys_alt;
  int32_t *__restrict__ vals = in_a ? d.plan.perm : d.tmp.vals_alt;
  int32_t *__restrict__ bag_tmp = d.tmp.bag_tmp, *__restrict__ counts = d.plan.counts;
  const int l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l <= num_bags) {
    bool bad;
    if (l < num_bags) bad = offsets[l] > offsets[l + 1] || offsets[l] < 0;
    else bad = offsets[num_bags] != (long long)nnz || offsets[0] != 0;
    if (bad) atomicOr(&counts[4], 2);
  }
  if (l >= nnz) return;
  long long row = indices[l];
  bool ok = row >= 0 && row < num_rows;
  if (ok && remap) {
    row = remap[row];
    ok = row >= 0 && row < num_rows;
  }
  if (!ok) atomicOr(&counts[4], 1);
  keys[l] = ok ? (int)row : sentinel;
  vals[l] = l;
  // largest b in [0, num_bags) with offsets[b] <= l  (empty bags share an offset and lose)
  int lo = 0, hi = num_bags;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (offsets[mid] <= (long long)l) lo = mid; else hi = mid;
  }
  bag_tmp[l] = lo;
}

// ------------------------------------------------------------------ LSD radix pass
// The three sorts of a plan: 0 = lookups by row, 1 = distinct rows by i3, 2 = distinct prefixes
// by i2.  (a) buffers hold the final result, (b) buffers are their ping-pong partners.
struct SortBufs {
  int32_t *ka, *va, *kb, *vb;
  const int32_t *count_ptr;
  int ntiles;
};
// `which` has to be a plain kernel argument: a variant that took it from the workgroup index (two
// sorts in one launch) was compiled to code that left one pointer of sort 2 at sort 1's value.
__device__ __forceinline__ SortBufs sort_bufs(const TTDev &d, int which) {
  SortBufs b;
  if (which == 0) {
    b.ka = d.plan.sorted_row; b.va = d.plan.perm; b.kb = d.tmp.keys_alt; b.vb = d.tmp.vals_alt;
    b.count_ptr = d.plan.counts + 3; b.ntiles = d.sort_tiles;
  } else if (which == 1) {
    b.ka = d.plan.i3_of_sorted; b.va = d.plan.rows_by_i3; b.kb = d.tmp.k3_alt; b.vb = d.tmp.v3_alt;
    b.count_ptr = d.plan.counts + 0;
    b.ntiles = (int)((d.plan.max_rows + TT_SORT_TILE - 1) / TT_SORT_TILE);
  } else {
    b.ka = d.tmp.k2; b.va = d.plan.prefs_by_i2; b.kb = d.tmp.k2_alt; b.vb = d.tmp.v2_alt;
    b.count_ptr = d.plan.counts + 1;
    b.ntiles = (int)((d.plan.max_prefixes + TT_SORT_TILE - 1) / TT_SORT_TILE);
  }
  return b;
}

template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_hist(TTArg<BATCHED> a, int which, int in_a, int shift, int bits) {
  const TTDev &d = a.get();
  const SortBufs sb = sort_bufs(d, which);
  const int ntiles = sb.ntiles;
  if ((int)blockIdx.x >= ntiles) return;  // uniform: this table has fewer tiles than the widest
  const int32_t *__restrict__ keys = in_a ? sb.ka : sb.kb;
  int32_t *__restrict__ hist = d.tmp.hist;
  __shared__ int h[1 << TT_SORT_MAX_BITS];
  const int nbins = 1 << bits, tile = blockIdx.x, count = *sb.count_ptr;
  for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) h[b] = 0;
  __syncthreads();
  const int base = tile * TT_SORT_TILE;
  if (base < count) {
#pragma unroll
    for (int i = 0; i < TT_SORT_ITEMS; ++i) {
      int pos = base + i * TT_BLOCK + threadIdx.x;
      if (pos < count) atomicAdd(&h[(keys[pos] >> shift) & (nbins - 1)], 1);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) hist[(size_t)tile * nbins + b] = h[b];  // [tile][bin]
}

// One workgroup per bin: exclusive scan of that bin's per-tile counts (a column of the [tile][bin]
// matrix), in place.  Only launched for sorts of many tiles; short sorts let every scatter
// workgroup add up its own column prefixes (one launch less per pass).
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_binscan(TTArg<BATCHED> a, int which, int nbins) {
  const TTDev &d = a.get();
  const int ntiles = sort_bufs(d, which).ntiles;
  int32_t *__restrict__ bin_total = d.tmp.bin_total;
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int32_t *col = d.tmp.hist + blockIdx.x;
  int carry = 0;
  for (int base = 0; base < ntiles; base += TT_BLOCK) {
    int t = base + threadIdx.x;
    int v = t < ntiles ? col[(size_t)t * nbins] : 0, total;
    int ex = tt_block_excl_scan(v, tmp, &total);
    if (t < ntiles) col[(size_t)t * nbins] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) bin_total[blockIdx.x] = carry;
}

// Orders the LDS accesses of the lanes of one wavefront (a wavefront executes them in program
// order; this keeps the compiler from moving them across).
__device__ __forceinline__ void tt_wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Stable scatter.  Wavefront w of a tile owns its keys [w*256, w*256 + 256) and ranks them in four
// rounds of 64 (position order), keeping per-digit running counts in its own row of wave_cnt; one
// scan over the four rows per digit then gives every wavefront its base inside the tile's run of
// that digit.  Equal digits keep their relative order: tiles in order, wavefronts in order, rounds
// in order, lanes in order.
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_scatter(TTArg<BATCHED> a, int which, int in_a, int shift, int bits, int self_scan) {
  const TTDev &d = a.get();
  const SortBufs sb = sort_bufs(d, which);
  const int ntiles = sb.ntiles;
  if ((int)blockIdx.x >= ntiles) return;  // uniform
  const int32_t *__restrict__ keys_in = in_a ? sb.ka : sb.kb, *__restrict__ vals_in = in_a ? sb.va : sb.vb;
  int32_t *__restrict__ keys_out = in_a ? sb.kb : sb.ka, *__restrict__ vals_out = in_a ? sb.vb : sb.va;
  const int32_t *__restrict__ count_ptr = sb.count_ptr, *__restrict__ hist = d.tmp.hist,
                *__restrict__ bin_total = d.tmp.bin_total;
  constexpr int MAXB = 1 << TT_SORT_MAX_BITS;
  constexpr int NW = TT_BLOCK / TT_WAVE;
  constexpr int PER = MAXB / TT_BLOCK;  // bins per thread: PER consecutive ones
  static_assert(PER == 4 && TT_SORT_ITEMS * TT_WAVE * NW == TT_SORT_TILE, "scatter geometry");
  __shared__ int gofs[MAXB];
  __shared__ int wave_cnt[NW][MAXB];
  __shared__ int tmp[NW + 1];
  const int nbins = 1 << bits, tile = blockIdx.x, count = *count_ptr;
  const int base = tile * TT_SORT_TILE;
  if (base >= count) return;  // uniform for the workgroup
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;

  // all keys and payloads of the tile are requested first (one memory round trip for the tile,
  // overlapped with the offset computation below)
  int keys_r[TT_SORT_ITEMS], vals_r[TT_SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int pos = base + (wave * TT_SORT_ITEMS + i) * TT_WAVE + lane;
    keys_r[i] = pos < count ? keys_in[pos] : 0;
    vals_r[i] = pos < count ? vals_in[pos] : 0;
  }

  // global offset of (bin, this tile) = exclusive scan of bin totals + tile prefix inside the bin
  {
    int loc[PER], pre[PER], sum = 0;
    const int b0 = threadIdx.x * PER;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      loc[k] = (b0 + k < nbins && !self_scan) ? bin_total[b0 + k] : 0;
      pre[k] = (b0 + k < nbins && !self_scan) ? hist[(size_t)tile * nbins + b0 + k] : 0;
    }
    if (self_scan) {  // raw per-tile counts: column totals and the prefix over the earlier tiles
      if (nbins >= PER) {  // rows are multiples of 16 bytes: one int4 per tile and thread
        if (b0 < nbins) {
#pragma unroll 16
          for (int t = 0; t < ntiles; ++t) {  // independent loads: sixteen tiles in flight
            const int4 v = *reinterpret_cast<const int4 *>(hist + (size_t)t * nbins + b0);
            const int m = t < tile ? -1 : 0;
            loc[0] += v.x; loc[1] += v.y; loc[2] += v.z; loc[3] += v.w;
            pre[0] += v.x & m; pre[1] += v.y & m; pre[2] += v.z & m; pre[3] += v.w & m;
          }
        }
      } else {
        for (int t = 0; t < ntiles; ++t)
#pragma unroll
          for (int k = 0; k < PER; ++k) {
            const int v = b0 + k < nbins ? hist[(size_t)t * nbins + b0 + k] : 0;
            loc[k] += v;
            pre[k] += t < tile ? v : 0;
          }
      }
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) sum += loc[k];
    int total, ex = tt_block_excl_scan(sum, tmp, &total);
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      if (b0 + k < nbins) {
        gofs[b0 + k] = ex + pre[k];
#pragma unroll
        for (int w = 0; w < NW; ++w) wave_cnt[w][b0 + k] = 0;
      }
      ex += loc[k];
    }
  }
  __syncthreads();

  int rank[TT_SORT_ITEMS], digit[TT_SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int pos = base + (wave * TT_SORT_ITEMS + i) * TT_WAVE + lane;
    const bool valid = pos < count;
    digit[i] = valid ? (keys_r[i] >> shift) & (nbins - 1) : 0;
    unsigned long long mask = __ballot(valid);  // lanes of this round with the same digit
    for (int b = 0; b < bits; ++b) {
      const bool bit = (digit[i] >> b) & 1;
      unsigned long long m = __ballot(valid && bit);
      mask &= bit ? m : ~m;
    }
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (TT_WAVE - lane));
    const int rank_in_round = __popcll(mask & lt);
    const int prev = valid ? wave_cnt[wave][digit[i]] : 0;  // this wavefront's earlier rounds
    tt_wave_lds_order();
    if (valid && rank_in_round == 0) wave_cnt[wave][digit[i]] = prev + __popcll(mask);
    tt_wave_lds_order();
    rank[i] = prev + rank_in_round;
  }
  __syncthreads();
  {  // per digit: counts of the wavefronts -> their bases inside the tile's run of the digit
    const int b0 = threadIdx.x * PER;
#pragma unroll
    for (int k = 0; k < PER; ++k)
      if (b0 + k < nbins) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const int c = wave_cnt[w][b0 + k];
          wave_cnt[w][b0 + k] = run;
          run += c;
        }
      }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int pos = base + (wave * TT_SORT_ITEMS + i) * TT_WAVE + lane;
    if (pos < count) {
      const int dst = gofs[digit[i]] + wave_cnt[wave][digit[i]] + rank[i];
      keys_out[dst] = keys_r[i];
      vals_out[dst] = vals_r[i];
    }
  }
}

// ------------------------------------------------------------------ distinct rows / prefixes
#define TT_UNIQ_ITEMS 4
#define TT_UNIQ_TILE (TT_BLOCK * TT_UNIQ_ITEMS)
#define TT_UNIQ_SELF_SCAN_TILES 1024  // up to this many tiles k_uniq_emit does without k_uniq_scan

__device__ __forceinline__ void head_flags(const int32_t *__restrict__ keys, int s, int nnz,
                                           int sentinel, int n3, int &hr, int &hp) {
  hr = hp = 0;
  if (s >= nnz) return;
  const int k = keys[s];
  if (k == sentinel) return;
  if (s == 0) { hr = hp = 1; return; }
  const int kp = keys[s - 1];
  hr = kp != k;
  hp = (kp / n3) != (k / n3);
}

template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_reduce(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const int nnz = d.nnz, sentinel = d.sh.sentinel, n3 = d.sh.n3;
  const int ntiles = (nnz + TT_UNIQ_TILE - 1) / TT_UNIQ_TILE;
  if ((int)blockIdx.x >= ntiles) return;  // uniform
  const int32_t *__restrict__ keys = d.plan.sorted_row;
  int32_t *__restrict__ tile_sums = d.tmp.tile_sums, *__restrict__ counts = d.plan.counts;
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int sr = 0, sp = 0;
  const int s0 = blockIdx.x * TT_UNIQ_TILE + threadIdx.x * TT_UNIQ_ITEMS;
#pragma unroll
  for (int i = 0; i < TT_UNIQ_ITEMS; ++i) {
    int hr, hp;
    head_flags(keys, s0 + i, nnz, sentinel, n3, hr, hp);
    sr += hr; sp += hp;
    const int s = s0 + i;
    // the last valid sorted position announces the number of valid lookups
    if (s < nnz && keys[s] != sentinel && (s == nnz - 1 || keys[s + 1] == sentinel))
      counts[2] = s + 1;
  }
  int tr, tp;
  tt_block_excl_scan(sr, tmp, &tr);
  tt_block_excl_scan(sp, tmp, &tp);
  if (threadIdx.x == 0) {
    tile_sums[blockIdx.x] = tr;
    tile_sums[ntiles + blockIdx.x] = tp;
  }
}

template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_scan(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const int ntiles = (d.nnz + TT_UNIQ_TILE - 1) / TT_UNIQ_TILE;
  int32_t *__restrict__ tile_sums = d.tmp.tile_sums, *__restrict__ counts = d.plan.counts,
          *__restrict__ row_seg = d.plan.row_seg, *__restrict__ pref_seg = d.plan.pref_seg;
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int carry[2] = {0, 0};
  for (int c = 0; c < 2; ++c) {
    int32_t *row = tile_sums + (size_t)c * ntiles;
    for (int base = 0; base < ntiles; base += TT_BLOCK) {
      int t = base + threadIdx.x;
      int v = t < ntiles ? row[t] : 0, total;
      int ex = tt_block_excl_scan(v, tmp, &total);
      if (t < ntiles) row[t] = carry[c] + ex;
      carry[c] += total;
    }
  }
  if (threadIdx.x == 0) {
    counts[0] = carry[0];
    counts[1] = carry[1];
    row_seg[carry[0]] = counts[2];
    pref_seg[carry[1]] = carry[0];
  }
}

// Also emits the keys of the two grouping sorts (i3 of every distinct row, i2 of every distinct
// prefix; a3 / a2: which of their ping-pong buffers the sorts start from).  With `self_scan` the
// tile sums are the raw ones of k_uniq_reduce: every workgroup adds up those of the earlier tiles
// itself and the last one writes the totals (one launch less than scanning them first).
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_emit(TTArg<BATCHED> a, int a3, int a2, int self_scan) {
  const TTDev &d = a.get();
  const int nnz = d.nnz, sentinel = d.sh.sentinel, n3 = d.sh.n3, n2 = d.sh.n2;
  const int ntiles = (nnz + TT_UNIQ_TILE - 1) / TT_UNIQ_TILE;
  if ((int)blockIdx.x >= ntiles) return;  // uniform
  const int32_t *__restrict__ keys = d.plan.sorted_row, *__restrict__ perm = d.plan.perm,
                *__restrict__ bag_tmp = d.tmp.bag_tmp, *__restrict__ tile_sums = d.tmp.tile_sums;
  int32_t *__restrict__ bag_of_sorted = d.plan.bag_of_sorted,
          *__restrict__ slot_of_sorted = d.plan.slot_of_sorted,
          *__restrict__ lookup2row = d.plan.lookup2row, *__restrict__ uniq_row = d.plan.uniq_row,
          *__restrict__ row_seg = d.plan.row_seg, *__restrict__ row2pref = d.plan.row2pref,
          *__restrict__ uniq_pref = d.plan.uniq_pref, *__restrict__ pref_seg = d.plan.pref_seg;
  int32_t *__restrict__ k3 = a3 ? d.plan.i3_of_sorted : d.tmp.k3_alt;
  int32_t *__restrict__ v3 = a3 ? d.plan.rows_by_i3 : d.tmp.v3_alt;
  int32_t *__restrict__ k2 = a2 ? d.tmp.k2 : d.tmp.k2_alt;
  int32_t *__restrict__ v2 = a2 ? d.plan.prefs_by_i2 : d.tmp.v2_alt;
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  const int s0 = blockIdx.x * TT_UNIQ_TILE + threadIdx.x * TT_UNIQ_ITEMS;
  int hr[TT_UNIQ_ITEMS], hp[TT_UNIQ_ITEMS], sr = 0, sp = 0;
#pragma unroll
  for (int i = 0; i < TT_UNIQ_ITEMS; ++i) {
    head_flags(keys, s0 + i, nnz, sentinel, n3, hr[i], hp[i]);
    sr += hr[i]; sp += hp[i];
  }
  int base_r, base_p;
  if (self_scan) {  // uniform
    int vr = 0, vp = 0;
    for (int t = threadIdx.x; t < (int)blockIdx.x; t += TT_BLOCK) {
      vr += tile_sums[t];
      vp += tile_sums[ntiles + t];
    }
    tt_block_excl_scan(vr, tmp, &base_r);
    tt_block_excl_scan(vp, tmp, &base_p);
  } else {
    base_r = tile_sums[blockIdx.x];
    base_p = tile_sums[ntiles + blockIdx.x];
  }
  int tot_r, tot_p;
  int er = tt_block_excl_scan(sr, tmp, &tot_r) + base_r;
  int ep = tt_block_excl_scan(sp, tmp, &tot_p) + base_p;
  if (self_scan && (int)blockIdx.x == ntiles - 1 && threadIdx.x == 0) {  // the totals
    int32_t *__restrict__ counts = d.plan.counts;
    counts[0] = base_r + tot_r;
    counts[1] = base_p + tot_p;
    row_seg[base_r + tot_r] = counts[2];
    pref_seg[base_p + tot_p] = base_r + tot_r;
  }
#pragma unroll
  for (int i = 0; i < TT_UNIQ_ITEMS; ++i) {
    const int s = s0 + i;
    if (s >= nnz) break;
    er += hr[i]; ep += hp[i];  // inclusive counts: slot = count - 1
    const int key = keys[s], l = perm[s];
    const bool valid = key != sentinel;
    const int slot_r = valid ? er - 1 : -1;
    bag_of_sorted[s] = bag_tmp[l];
    slot_of_sorted[s] = slot_r;
    lookup2row[l] = slot_r;
    if (hr[i]) {
      uniq_row[slot_r] = key;
      row_seg[slot_r] = s;
      row2pref[slot_r] = ep - 1;
      k3[slot_r] = key % n3;
      v3[slot_r] = slot_r;
    }
    if (hp[i]) {
      uniq_pref[ep - 1] = key / n3;
      pref_seg[ep - 1] = slot_r;
      k2[ep - 1] = (key / n3) % n2;
      v2[ep - 1] = ep - 1;
    }
  }
}

// ------------------------------------------------------------------ groupings by i3 / i2 / i1
// seg[t] = first position of the sorted keys whose key is >= t, for t = 0..nkeys: the thread of
// position u fills the entries between its predecessor's key and its own (one memory round trip
// per thread instead of a binary search), the thread of the last position also the tail.
__device__ __forceinline__ void seg_starts(const int32_t *__restrict__ keys, int div, int count, int nkeys,
                                           int32_t *__restrict__ seg, int u) {
  if (count == 0) {
    if (u <= nkeys) seg[u] = 0;
    return;
  }
  if (u >= count) return;
  const int key = keys[u] / div, prev = u > 0 ? keys[u - 1] / div : -1;
  for (int t = prev + 1; t <= key; ++t) seg[t] = u;
  if (u == count - 1)
    for (int t = key + 1; t <= nkeys; ++t) seg[t] = count;
}

template <bool BATCHED>
__global__ void k_seg_bounds(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const int32_t *__restrict__ counts = d.plan.counts;
  const int ur = counts[0], up = counts[1];
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  seg_starts(d.plan.i3_of_sorted, 1, ur, d.sh.n3, d.plan.i3_seg, u);
  seg_starts(d.tmp.k2, 1, up, d.sh.n2, d.plan.i2_seg, u);
  seg_starts(d.plan.uniq_pref, d.sh.n2, up, d.sh.n1, d.plan.i1_seg, u);
  if (u < up) {  // what the matrix-core kernels need to know about the u-th prefix in i2 order
    const int q = d.plan.prefs_by_i2[u], u0 = d.plan.pref_seg[q];
    reinterpret_cast<int4 *>(d.plan.pref_meta)[u] = make_int4(d.plan.uniq_pref[q] / d.sh.n2, u0, d.plan.pref_seg[q + 1] - u0, q);
  }
}

// Running count of TT_MP-prefix chunks per i2 (single workgroup; n2 may exceed the block size).
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_chunk_offsets(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const int32_t *__restrict__ i2_seg = d.plan.i2_seg;
  const int n2 = d.sh.n2;
  int32_t *__restrict__ chunk_off = d.plan.i2_chunk_off, *__restrict__ counts = d.plan.counts;
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int carry = 0;
  for (int base = 0; base < n2; base += TT_BLOCK) {
    const int t = base + threadIdx.x;
    int v = 0, total;
    if (t < n2) v = (i2_seg[t + 1] - i2_seg[t] + TT_MP - 1) / TT_MP;
    const int ex = tt_block_excl_scan(v, tmp, &total);
    if (t < n2) chunk_off[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    chunk_off[n2] = carry;
    counts[5] = carry;
  }
  __syncthreads();  // the offsets written above are read back below (same workgroup)
  int4 *__restrict__ chunk_rec = reinterpret_cast<int4 *>(d.plan.chunk_i2);  // i2, first prefix position, prefixes, 0
  for (int t = threadIdx.x; t < n2; t += TT_BLOCK) {
    const int c0 = chunk_off[t], c1 = t + 1 < n2 ? chunk_off[t + 1] : carry;
    const int first = i2_seg[t], end = i2_seg[t + 1];
    for (int c = c0; c < c1; ++c) {
      const int cs = first + (c - c0) * TT_MP;
      chunk_rec[c] = make_int4(t, cs, (end - cs) < TT_MP ? (end - cs) : TT_MP, 0);
    }
  }
}

int bit_length(long long v) {
  int b = 0;
  while (v > 0) { ++b; v >>= 1; }
  return b;
}

#ifndef TT_SELF_SCAN_TILES
#define TT_SELF_SCAN_TILES 64  // sorts of at most this many tiles skip the bin-scan launch
#endif
struct RadixPlan { int passes; int bits_per_pass; };
RadixPlan radix_plan(int key_bits) {
  RadixPlan p;
  p.passes = (key_bits + TT_SORT_MAX_BITS - 1) / TT_SORT_MAX_BITS;
  p.bits_per_pass = p.passes ? (key_bits + p.passes - 1) / p.passes : 0;
  return p;
}

// One of the three sorts, for every table of the batch, with the same pass structure (so that a
// pass is one launch): key_bits is the widest key of the batch.  The input must sit in the (a)
// buffers when the number of passes is even and in (b) when it is odd; the result lands in (a).
tt_status radix_sort(const TTBatch &b, int which, int max_tiles, int key_bits, hipStream_t s) {
  const RadixPlan rp = radix_plan(key_bits);
  if (max_tiles == 0) return TT_OK;
  int in_a = (rp.passes % 2) == 0;
  int shift = 0;
  for (int p = 0; p < rp.passes; ++p) {
    const int bits = (key_bits - shift) < rp.bits_per_pass ? (key_bits - shift) : rp.bits_per_pass;
    const int self_scan = max_tiles <= TT_SELF_SCAN_TILES ? 1 : 0;
    TT_LAUNCH(k_radix_hist, max_tiles, TT_BLOCK, 0, s, b, which, in_a, shift, bits);
    if (!self_scan) TT_LAUNCH(k_radix_binscan, 1 << bits, TT_BLOCK, 0, s, b, which, 1 << bits);
    {
      TTProfScope prof(which == 0 ? &b.host[0].plan : nullptr, TT_KERNEL_SORT_SCATTER, s);
      TT_LAUNCH(k_radix_scatter, max_tiles, TT_BLOCK, 0, s, b, which, in_a, shift, bits, self_scan);
    }
    shift += bits;
    in_a = !in_a;
  }
  return tt_launch_status();
}

}  // namespace

size_t tt_sort_tmp_bytes(int64_t nnz, int64_t max_rows, int64_t max_prefixes) {
  const size_t ntiles = (size_t)tt_ceil_div(nnz, TT_SORT_TILE) + 1;
  const size_t utiles = (size_t)tt_ceil_div(nnz, TT_UNIQ_TILE) + 1;
  size_t ints = 3 * (size_t)nnz + 2 * (size_t)max_rows + 3 * (size_t)max_prefixes +
                ((size_t)1 << TT_SORT_MAX_BITS) * ntiles + ((size_t)1 << TT_SORT_MAX_BITS) +
                2 * utiles;
  return (ints + 64 * 12) * sizeof(int32_t);
}

TTSortTmp tt_sort_tmp_view(const tt_plan *plan) {
  TTSortTmp t;
  const size_t nnz = (size_t)plan->nnz, mr = (size_t)plan->max_rows,
               mp = (size_t)plan->max_prefixes;
  const size_t ntiles = (size_t)tt_ceil_div(plan->nnz, TT_SORT_TILE) + 1;
  int32_t *p = (int32_t *)plan->sort_tmp;
  auto take = [&](size_t count) {
    int32_t *q = p;
    p += (count + 63) / 64 * 64;  // keep every array 256-byte aligned
    return q;
  };
  t.keys_alt = take(nnz);
  t.vals_alt = take(nnz);
  t.bag_tmp = take(nnz);
  t.k3_alt = take(mr);
  t.v3_alt = take(mr);
  t.k2 = take(mp);
  t.k2_alt = take(mp);
  t.v2_alt = take(mp);
  t.hist = take(((size_t)1 << TT_SORT_MAX_BITS) * ntiles);
  t.bin_total = take((size_t)1 << TT_SORT_MAX_BITS);
  t.tile_sums = take(2 * ((size_t)tt_ceil_div(plan->nnz, TT_UNIQ_TILE) + 1));
  return t;
}

tt_status ttk_reorder(const TTBatch &b, hipStream_t s) {
  TT_LAUNCH(k_init_counts, 1, 64, 0, s, b);

  // main sort: keys in [0, sentinel]
  const int key_bits = bit_length(tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.sentinel; }));
  const int in_a = (radix_plan(key_bits).passes % 2) == 0;
  const long long cover = tt_batch_max(b, [](const TTDev &d) {
    return (long long)(d.nnz > d.num_bags + 1 ? d.nnz : d.num_bags + 1); });
  TT_LAUNCH(k_extract_keys, tt_ceil_div(cover, TT_BLOCK), TT_BLOCK, 0, s, b, in_a);
  const int tiles0 = (int)tt_batch_max(b, [](const TTDev &d) { return (long long)d.sort_tiles; });
  tt_status st = radix_sort(b, 0, tiles0, key_bits, s);
  if (st != TT_OK) return st;

  // distinct rows and prefixes
  const int utiles = (int)tt_batch_max(b, [](const TTDev &d) {
    return (long long)tt_ceil_div(d.nnz, TT_UNIQ_TILE); });
  // groupings: distinct rows by i3, distinct prefixes by i2 (stable), i1 ranges
  const int bits3 = bit_length(tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n3 - 1; }));
  const int bits2 = bit_length(tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n2 - 1; }));
  const int a3 = (radix_plan(bits3).passes % 2) == 0, a2 = (radix_plan(bits2).passes % 2) == 0;
  const long long max_rows = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_rows; });
  const long long max_pref = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_prefixes; });
  // short inputs: every emit workgroup adds up the earlier tiles' sums itself (no scan launch)
  const int uniq_self = (utiles > 0 && utiles <= TT_UNIQ_SELF_SCAN_TILES) ? 1 : 0;
  if (utiles > 0) TT_LAUNCH(k_uniq_reduce, utiles, TT_BLOCK, 0, s, b);
  if (!uniq_self) TT_LAUNCH(k_uniq_scan, 1, TT_BLOCK, 0, s, b);
  if (utiles > 0) TT_LAUNCH(k_uniq_emit, utiles, TT_BLOCK, 0, s, b, a3, a2, uniq_self);
  if (max_rows > 0) {
    st = radix_sort(b, 1, tt_ceil_div(max_rows, TT_SORT_TILE), bits3, s);
    if (st != TT_OK) return st;
    st = radix_sort(b, 2, tt_ceil_div(max_pref, TT_SORT_TILE), bits2, s);
    if (st != TT_OK) return st;
  }
  // one thread per sorted position (and at least one per segment boundary when a count is zero)
  const long long nmax = tt_batch_max(b, [](const TTDev &d) {
    long long m = d.sh.n1 > d.sh.n2 ? d.sh.n1 : d.sh.n2;
    m = m > d.sh.n3 ? m : (long long)d.sh.n3;
    m += 1;
    return m > d.plan.max_rows ? m : (long long)d.plan.max_rows; });
  TT_LAUNCH(k_seg_bounds, tt_ceil_div(nmax, TT_BLOCK), TT_BLOCK, 0, s, b);
  TT_LAUNCH(k_chunk_offsets, 1, TT_BLOCK, 0, s, b);
  return tt_launch_status();
}
