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
__global__ void k_init_counts(int32_t *counts, int nnz) {
  if (threadIdx.x < 16) counts[threadIdx.x] = (threadIdx.x == 3) ? nnz : 0;
}

// One thread per lookup: validate, apply the optional bijection, emit (row, position) and the
// bag holding the position.  Threads b <= num_bags also validate the CSR offsets.
__global__ void k_extract_keys(const int64_t *__restrict__ indices,
                               const int64_t *__restrict__ offsets,
                               const int64_t *__restrict__ remap, int nnz, int num_bags,
                               long long num_rows, int sentinel, int32_t *__restrict__ keys,
                               int32_t *__restrict__ vals, int32_t *__restrict__ bag_tmp,
                               int32_t *__restrict__ counts) {
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
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_hist(const int32_t *__restrict__ keys, const int32_t *__restrict__ count_ptr, int shift,
             int bits, int ntiles, int32_t *__restrict__ hist) {
  __shared__ int h[1 << TT_SORT_MAX_BITS];
  const int nbins = 1 << bits, tile = blockIdx.x, count = *count_ptr;
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
  for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) hist[(size_t)b * ntiles + tile] = h[b];
}

// One workgroup per bin: exclusive scan of that bin's per-tile counts, in place.
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_binscan(int32_t *__restrict__ hist, int ntiles, int32_t *__restrict__ bin_total) {
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int32_t *row = hist + (size_t)blockIdx.x * ntiles;
  int carry = 0;
  for (int base = 0; base < ntiles; base += TT_BLOCK) {
    int t = base + threadIdx.x;
    int v = t < ntiles ? row[t] : 0, total;
    int ex = tt_block_excl_scan(v, tmp, &total);
    if (t < ntiles) row[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) bin_total[blockIdx.x] = carry;
}

// Stable scatter: elements of a tile are ranked in tile order (round i, thread t) so that equal
// digits keep their relative order.
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_scatter(const int32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in,
                int32_t *__restrict__ keys_out, int32_t *__restrict__ vals_out,
                const int32_t *__restrict__ count_ptr, int shift, int bits, int ntiles,
                const int32_t *__restrict__ hist, const int32_t *__restrict__ bin_total) {
  constexpr int MAXB = 1 << TT_SORT_MAX_BITS;
  constexpr int NW = TT_BLOCK / TT_WAVE;
  __shared__ int gofs[MAXB];
  __shared__ int run[MAXB];
  __shared__ int wave_cnt[NW][MAXB];
  __shared__ int tmp[NW + 1];
  const int nbins = 1 << bits, tile = blockIdx.x, count = *count_ptr;
  const int base = tile * TT_SORT_TILE;
  if (base >= count) return;  // uniform for the workgroup
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;

  // global offset of (bin, this tile) = exclusive scan of bin totals + tile prefix inside the bin
  {
    constexpr int PER = MAXB / TT_BLOCK;
    int loc[PER], sum = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      int b = threadIdx.x * PER + k;
      loc[k] = b < nbins ? bin_total[b] : 0;
      sum += loc[k];
    }
    int total, ex = tt_block_excl_scan(sum, tmp, &total);
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      int b = threadIdx.x * PER + k;
      if (b < nbins) {
        gofs[b] = ex + hist[(size_t)b * ntiles + tile];
        run[b] = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) wave_cnt[w][b] = 0;
      }
      ex += loc[k];
    }
  }
  __syncthreads();

  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int pos = base + i * TT_BLOCK + threadIdx.x;
    const bool valid = pos < count;
    int key = 0, val = 0, digit = 0;
    if (valid) {
      key = keys_in[pos];
      val = vals_in[pos];
      digit = (key >> shift) & (nbins - 1);
    }
    unsigned long long mask = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
      const bool bit = (digit >> b) & 1;
      unsigned long long m = __ballot(valid && bit);
      mask &= bit ? m : ~m;
    }
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (TT_WAVE - lane));
    const int rank_in_wave = __popcll(mask & lt);
    if (valid && rank_in_wave == 0) wave_cnt[wave][digit] = __popcll(mask);
    __syncthreads();
    int my = 0;
    if (valid) {
      my = run[digit] + rank_in_wave;
      for (int w = 0; w < wave; ++w) my += wave_cnt[w][digit];
    }
    __syncthreads();
    for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) {
      int add = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) { add += wave_cnt[w][b]; wave_cnt[w][b] = 0; }
      run[b] += add;
    }
    if (valid) {
      const int dst = gofs[digit] + my;
      keys_out[dst] = key;
      vals_out[dst] = val;
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------ distinct rows / prefixes
#define TT_UNIQ_ITEMS 4
#define TT_UNIQ_TILE (TT_BLOCK * TT_UNIQ_ITEMS)

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

__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_reduce(const int32_t *__restrict__ keys, int nnz, int sentinel, int n3, int ntiles,
              int32_t *__restrict__ tile_sums, int32_t *__restrict__ counts) {
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

__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_scan(int32_t *__restrict__ tile_sums, int ntiles, int32_t *__restrict__ counts,
            int32_t *__restrict__ row_seg, int32_t *__restrict__ pref_seg) {
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

__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_emit(const int32_t *__restrict__ keys, const int32_t *__restrict__ perm,
            const int32_t *__restrict__ bag_tmp, int nnz, int sentinel, int n3, int ntiles,
            const int32_t *__restrict__ tile_sums, int32_t *__restrict__ bag_of_sorted,
            int32_t *__restrict__ slot_of_sorted, int32_t *__restrict__ lookup2row,
            int32_t *__restrict__ uniq_row, int32_t *__restrict__ row_seg,
            int32_t *__restrict__ row2pref, int32_t *__restrict__ uniq_pref,
            int32_t *__restrict__ pref_seg) {
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  const int s0 = blockIdx.x * TT_UNIQ_TILE + threadIdx.x * TT_UNIQ_ITEMS;
  int hr[TT_UNIQ_ITEMS], hp[TT_UNIQ_ITEMS], sr = 0, sp = 0;
#pragma unroll
  for (int i = 0; i < TT_UNIQ_ITEMS; ++i) {
    head_flags(keys, s0 + i, nnz, sentinel, n3, hr[i], hp[i]);
    sr += hr[i]; sp += hp[i];
  }
  int tot;
  int er = tt_block_excl_scan(sr, tmp, &tot) + tile_sums[blockIdx.x];
  int ep = tt_block_excl_scan(sp, tmp, &tot) + tile_sums[ntiles + blockIdx.x];
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
    }
    if (hp[i]) {
      uniq_pref[ep - 1] = key / n3;
      pref_seg[ep - 1] = slot_r;
    }
  }
}

// ------------------------------------------------------------------ groupings by i3 / i2 / i1
__global__ void k_group_keys(const int32_t *__restrict__ counts,
                             const int32_t *__restrict__ uniq_row, int n3,
                             int32_t *__restrict__ k3, int32_t *__restrict__ v3,
                             const int32_t *__restrict__ uniq_pref, int n2,
                             int32_t *__restrict__ k2, int32_t *__restrict__ v2) {
  const int ur = counts[0], up = counts[1];
  for (int u = blockIdx.x * blockDim.x + threadIdx.x; u < ur; u += gridDim.x * blockDim.x) {
    k3[u] = uniq_row[u] % n3;
    v3[u] = u;
    if (u < up) {
      k2[u] = uniq_pref[u] % n2;
      v2[u] = u;
    }
  }
}

__device__ __forceinline__ int lower_bound_div(const int32_t *__restrict__ a, int count, int div,
                                               int value) {
  int lo = 0, hi = count;  // first position with a[pos]/div >= value
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (a[mid] / div < value) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__global__ void k_seg_bounds(const int32_t *__restrict__ counts,
                             const int32_t *__restrict__ k3_sorted, int n3,
                             int32_t *__restrict__ i3_seg, const int32_t *__restrict__ k2_sorted,
                             int n2, int32_t *__restrict__ i2_seg,
                             const int32_t *__restrict__ uniq_pref, int n1,
                             int32_t *__restrict__ i1_seg) {
  const int ur = counts[0], up = counts[1];
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t <= n3) i3_seg[t] = lower_bound_div(k3_sorted, ur, 1, t);
  if (t <= n2) i2_seg[t] = lower_bound_div(k2_sorted, up, 1, t);
  if (t <= n1) i1_seg[t] = lower_bound_div(uniq_pref, up, n2, t);
}

// Running count of TT_MP-prefix chunks per i2 (single workgroup; n2 may exceed the block size).
__global__ void __launch_bounds__(TT_BLOCK)
k_chunk_offsets(const int32_t *__restrict__ i2_seg, int n2, int32_t *__restrict__ chunk_off,
                int32_t *__restrict__ counts) {
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
}

int bit_length(long long v) {
  int b = 0;
  while (v > 0) { ++b; v >>= 1; }
  return b;
}

struct RadixPlan { int passes; int bits_per_pass; };
RadixPlan radix_plan(int key_bits) {
  RadixPlan p;
  p.passes = (key_bits + TT_SORT_MAX_BITS - 1) / TT_SORT_MAX_BITS;
  p.bits_per_pass = p.passes ? (key_bits + p.passes - 1) / p.passes : 0;
  return p;
}

// Sort (keys, vals) of *count_ptr (<= max_count) elements.  The input must sit in
// (a) when the number of passes is even and in (b) when it is odd; the result lands in (a).
tt_status radix_sort(int32_t *keys_a, int32_t *vals_a, int32_t *keys_b, int32_t *vals_b,
                     const int32_t *count_ptr, int64_t max_count, int key_bits,
                     const TTSortTmp &tmp, hipStream_t s, const tt_plan *prof_plan = nullptr) {
  const RadixPlan rp = radix_plan(key_bits);
  const int ntiles = tt_ceil_div(max_count, TT_SORT_TILE);
  if (ntiles == 0) return TT_OK;
  bool in_a = (rp.passes % 2) == 0;
  int shift = 0;
  for (int p = 0; p < rp.passes; ++p) {
    const int bits = (key_bits - shift) < rp.bits_per_pass ? (key_bits - shift) : rp.bits_per_pass;
    int32_t *ki = in_a ? keys_a : keys_b, *vi = in_a ? vals_a : vals_b;
    int32_t *ko = in_a ? keys_b : keys_a, *vo = in_a ? vals_b : vals_a;
    hipLaunchKernelGGL(k_radix_hist, dim3(ntiles), dim3(TT_BLOCK), 0, s, ki, count_ptr, shift,
                       bits, ntiles, tmp.hist);
    hipLaunchKernelGGL(k_radix_binscan, dim3(1 << bits), dim3(TT_BLOCK), 0, s, tmp.hist, ntiles,
                       tmp.bin_total);
    {
      TTProfScope prof(prof_plan, TT_KERNEL_SORT_SCATTER, s);
      hipLaunchKernelGGL(k_radix_scatter, dim3(ntiles), dim3(TT_BLOCK), 0, s, ki, vi, ko, vo,
                         count_ptr, shift, bits, ntiles, tmp.hist, tmp.bin_total);
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

tt_status ttk_reorder(const TTShape &sh, const int64_t *indices, const int64_t *offsets,
                      int64_t nnz64, int64_t num_bags64, const int64_t *remap,
                      const tt_plan *plan, hipStream_t s) {
  const int nnz = (int)nnz64, num_bags = (int)num_bags64;
  const TTSortTmp tmp = tt_sort_tmp_view(plan);
  hipLaunchKernelGGL(k_init_counts, dim3(1), dim3(64), 0, s, plan->counts, nnz);

  // main sort: keys in [0, sentinel]
  const int key_bits = bit_length(sh.sentinel);
  const bool in_a = (radix_plan(key_bits).passes % 2) == 0;
  int32_t *k0 = in_a ? plan->sorted_row : tmp.keys_alt, *v0 = in_a ? plan->perm : tmp.vals_alt;
  const int cover = (nnz > num_bags + 1 ? nnz : num_bags + 1);
  hipLaunchKernelGGL(k_extract_keys, dim3(tt_ceil_div(cover, TT_BLOCK)), dim3(TT_BLOCK), 0, s,
                     indices, offsets, remap, nnz, num_bags, sh.num_rows, sh.sentinel, k0, v0,
                     tmp.bag_tmp, plan->counts);
  tt_status st = radix_sort(plan->sorted_row, plan->perm, tmp.keys_alt, tmp.vals_alt,
                            plan->counts + 3, nnz, key_bits, tmp, s, plan);
  if (st != TT_OK) return st;

  // distinct rows and prefixes
  const int utiles = tt_ceil_div(nnz, TT_UNIQ_TILE);
  if (utiles > 0)
    hipLaunchKernelGGL(k_uniq_reduce, dim3(utiles), dim3(TT_BLOCK), 0, s, plan->sorted_row, nnz,
                       sh.sentinel, sh.n3, utiles, tmp.tile_sums, plan->counts);
  hipLaunchKernelGGL(k_uniq_scan, dim3(1), dim3(TT_BLOCK), 0, s, tmp.tile_sums, utiles,
                     plan->counts, plan->row_seg, plan->pref_seg);
  if (utiles > 0)
    hipLaunchKernelGGL(k_uniq_emit, dim3(utiles), dim3(TT_BLOCK), 0, s, plan->sorted_row,
                       plan->perm, tmp.bag_tmp, nnz, sh.sentinel, sh.n3, utiles, tmp.tile_sums,
                       plan->bag_of_sorted, plan->slot_of_sorted, plan->lookup2row,
                       plan->uniq_row, plan->row_seg, plan->row2pref, plan->uniq_pref,
                       plan->pref_seg);

  // groupings: distinct rows by i3, distinct prefixes by i2 (stable), i1 ranges
  const int bits3 = bit_length(sh.n3 - 1), bits2 = bit_length(sh.n2 - 1);
  const bool a3 = (radix_plan(bits3).passes % 2) == 0, a2 = (radix_plan(bits2).passes % 2) == 0;
  int32_t *k3in = a3 ? plan->i3_of_sorted : tmp.k3_alt, *v3in = a3 ? plan->rows_by_i3 : tmp.v3_alt;
  int32_t *k2in = a2 ? tmp.k2 : tmp.k2_alt, *v2in = a2 ? plan->prefs_by_i2 : tmp.v2_alt;
  if (plan->max_rows > 0) {
    int blocks = tt_ceil_div(plan->max_rows, TT_BLOCK);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_group_keys, dim3(blocks), dim3(TT_BLOCK), 0, s, plan->counts,
                       plan->uniq_row, sh.n3, k3in, v3in, plan->uniq_pref, sh.n2, k2in, v2in);
    st = radix_sort(plan->i3_of_sorted, plan->rows_by_i3, tmp.k3_alt, tmp.v3_alt, plan->counts + 0,
                    plan->max_rows, bits3, tmp, s);
    if (st != TT_OK) return st;
    st = radix_sort(tmp.k2, plan->prefs_by_i2, tmp.k2_alt, tmp.v2_alt, plan->counts + 1,
                    plan->max_prefixes, bits2, tmp, s);
    if (st != TT_OK) return st;
  }
  int nmax = sh.n1 > sh.n2 ? sh.n1 : sh.n2;
  if (sh.n3 > nmax) nmax = sh.n3;
  hipLaunchKernelGGL(k_seg_bounds, dim3(tt_ceil_div(nmax + 1, TT_BLOCK)), dim3(TT_BLOCK), 0, s,
                     plan->counts, plan->i3_of_sorted, sh.n3, plan->i3_seg, tmp.k2, sh.n2,
                     plan->i2_seg, plan->uniq_pref, sh.n1, plan->i1_seg);
  hipLaunchKernelGGL(k_chunk_offsets, dim3(1), dim3(TT_BLOCK), 0, s, plan->i2_seg, sh.n2,
                     plan->i2_chunk_off, plan->counts);
  return tt_launch_status();
}
