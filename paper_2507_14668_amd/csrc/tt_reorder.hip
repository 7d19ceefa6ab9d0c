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
// Errors only the device can see.  They are reported with atomics on the plan's status word, so
// they are checked in the SECOND kernel of the plan (the first one initialises that word).
__device__ __forceinline__ void check_offsets(const TTDev &d, int l) {
  const int64_t *__restrict__ offsets = d.offsets;
  const int num_bags = d.num_bags;
  if (l > num_bags) return;
  bool bad;
  if (l < num_bags) bad = offsets[l] > offsets[l + 1] || offsets[l] < 0;
  else bad = offsets[num_bags] != (long long)d.nnz || offsets[0] != 0;
  if (bad) atomicOr(&d.plan.counts[4], 2);
}

// First kernel of a plan.  Workgroup 0 initialises the counters; every workgroup takes one sort
// tile of lookups: validate, apply the optional bijection, emit (row, position) and the bag holding
// the position, and count the first radix digit of the tile's keys (so that the first sort pass
// needs no histogram launch).  An invalid lookup gets the sentinel key n1*n2*n3.
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_extract_keys(TTArg<BATCHED> a, int in_a, int bits, int passes) {
  const TTDev &d = a.get();
  const int64_t *__restrict__ indices = d.indices, *__restrict__ offsets = d.offsets,
                *__restrict__ remap = d.remap;
  const int nnz = d.nnz, num_bags = d.num_bags, sentinel = d.sh.sentinel;
  const long long num_rows = d.sh.num_rows;
  int32_t *__restrict__ keys = in_a ? d.plan.sorted_row : d.tmp.keys_alt;
  int32_t *__restrict__ vals = in_a ? d.plan.perm : d.tmp.vals_alt;
  int32_t *__restrict__ bag_tmp = d.tmp.bag_tmp, *__restrict__ hist = d.tmp.hist;
  const size_t hist_stride = ((size_t)1 << TT_SORT_MAX_BITS) * ((size_t)d.sort_tiles + 1);
  if (blockIdx.x == 0) {
    if (threadIdx.x < 16) d.plan.counts[threadIdx.x] = (threadIdx.x == 3) ? nnz : 0;
    // a table without lookups has no workgroup that would write the terminal segment entries
    if (threadIdx.x == 16) d.plan.row_seg[0] = 0;
    if (threadIdx.x == 17) d.plan.pref_seg[0] = 0;
  }
  if ((int)blockIdx.x >= d.sort_tiles) return;  // uniform: a table of the batch with fewer tiles
  __shared__ int h[1 << TT_SORT_MAX_BITS];
  const int nbins = 1 << bits;
  for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) h[b] = 0;
  __syncthreads();
  // the thread's four lookups go through every step together, so that their loads overlap
  long long row[TT_SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int l = blockIdx.x * TT_SORT_TILE + i * TT_BLOCK + threadIdx.x;
    row[i] = l < nnz ? indices[l] : -1;
  }
  if (remap) {
#pragma unroll
    for (int i = 0; i < TT_SORT_ITEMS; ++i)
      if (row[i] >= 0 && row[i] < num_rows) row[i] = remap[row[i]];
  }
  // largest b in [0, num_bags) with offsets[b] <= l  (empty bags share an offset and lose)
  int lo[TT_SORT_ITEMS], hi[TT_SORT_ITEMS];
  bool searching = false;
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int l = blockIdx.x * TT_SORT_TILE + i * TT_BLOCK + threadIdx.x;
    lo[i] = 0; hi[i] = num_bags;
    if (l < nnz && l < num_bags && offsets[l] == (long long)l && offsets[l + 1] > (long long)l) {
      lo[i] = l; hi[i] = l + 1;  // bag b starts at lookup b (every earlier bag holds one lookup): no search
    }
    if (l >= nnz) hi[i] = lo[i] + 1;  // no lookup: nothing to find
    searching |= hi[i] - lo[i] > 1;
  }
  // Multi-lookup bags.  The tile's lookups are consecutive, so their bags start at the bag of the
  // tile's first lookup: the workgroup finds that bag with a 256-ary search (two rounds of one probe
  // per thread for 65 536 bags, instead of sixteen dependent halving steps per thread), stages the
  // next TT_SORT_TILE + 1 offsets in LDS and every thread bisects there.  Only a thread whose bag lies
  // beyond the staged window (more than a tile's worth of bags, i.e. runs of empty bags) goes on
  // halving in memory.  With offsets that are not monotone the searches still stay inside
  // [0, num_bags]; the offsets check reports them.
  __shared__ long long s_off[TT_SORT_TILE + 1];
  __shared__ int s_cnt[TT_BLOCK / TT_WAVE], s_any;
  if (threadIdx.x == 0) s_any = 0;
  __syncthreads();
  if (searching) s_any = 1;
  __syncthreads();
  if (s_any) {  // uniform
    const long long first = (long long)blockIdx.x * TT_SORT_TILE;
    int wlo = 0, whi = num_bags;  // the bag of lookup `first` is in [wlo, whi)
    while (whi - wlo > 1) {       // uniform
      const int step = (whi - wlo + TT_BLOCK) / (TT_BLOCK + 1);  // probes wlo + (t+1)*step, t = thread
      const long long q = (long long)wlo + (long long)(threadIdx.x + 1) * step;
      const bool le = q < whi && offsets[q] <= first;
      const unsigned long long m = __ballot(le);
      if ((threadIdx.x & (TT_WAVE - 1)) == 0) s_cnt[threadIdx.x / TT_WAVE] = __popcll(m);
      __syncthreads();
      int cnt = 0;
#pragma unroll
      for (int w = 0; w < TT_BLOCK / TT_WAVE; ++w) cnt += s_cnt[w];
      __syncthreads();
      // monotone offsets: the probes that are <= first are the first `cnt` ones
      const long long nlo = (long long)wlo + (long long)cnt * step, nhi = nlo + step;
      wlo = (int)nlo;
      whi = nhi < whi ? (int)nhi : whi;
    }
    const int wcount = (num_bags + 1 - wlo) < (TT_SORT_TILE + 1) ? (num_bags + 1 - wlo) : (TT_SORT_TILE + 1);
    for (int e = threadIdx.x; e < wcount; e += TT_BLOCK) s_off[e] = offsets[wlo + e];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TT_SORT_ITEMS; ++i) {
      const int l = blockIdx.x * TT_SORT_TILE + i * TT_BLOCK + threadIdx.x;
      if (hi[i] - lo[i] <= 1) continue;
      if (s_off[wcount - 1] <= (long long)l && wlo + wcount - 1 < num_bags) {
        lo[i] = wlo + wcount - 1;  // beyond the window: go on in memory
        continue;
      }
      int a = 0, b = wcount - 1;  // s_off[a] <= l is assumed, the answer is in [a, b)
      if (s_off[b] <= (long long)l) b = wcount;  // the last bag of the table
      while (b - a > 1) {
        const int mid = (a + b) >> 1;
        if (s_off[mid] <= (long long)l) a = mid; else b = mid;
      }
      lo[i] = wlo + a < num_bags ? wlo + a : num_bags - 1;
      hi[i] = lo[i] + 1;
    }
    searching = false;
#pragma unroll
    for (int i = 0; i < TT_SORT_ITEMS; ++i) searching |= hi[i] - lo[i] > 1;
  }
  while (searching) {  // one halving step for all four per round
    searching = false;
#pragma unroll
    for (int i = 0; i < TT_SORT_ITEMS; ++i) {
      const int l = blockIdx.x * TT_SORT_TILE + i * TT_BLOCK + threadIdx.x;
      if (hi[i] - lo[i] > 1) {
        const int mid = (lo[i] + hi[i]) >> 1;
        if (offsets[mid] <= (long long)l) lo[i] = mid; else hi[i] = mid;
        searching |= hi[i] - lo[i] > 1;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {
    const int l = blockIdx.x * TT_SORT_TILE + i * TT_BLOCK + threadIdx.x;
    if (l >= nnz) continue;
    const bool ok = row[i] >= 0 && row[i] < num_rows;
    const int key = ok ? (int)row[i] : sentinel;
    keys[l] = key;
    vals[l] = l;
    atomicAdd(&h[key & (nbins - 1)], 1);
    bag_tmp[l] = lo[i];
  }
  __syncthreads();
  for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) hist[(size_t)blockIdx.x * nbins + b] = h[b];  // [tile][bin]
  // the scatter of pass p counts the digits of pass p + 1 into that pass's array: clear this tile's rows
  for (int p = 1; p < passes; ++p)
    for (int b = threadIdx.x; b < (1 << TT_SORT_MAX_BITS); b += TT_BLOCK)
      hist[p * hist_stride + (size_t)blockIdx.x * (1 << TT_SORT_MAX_BITS) + b] = 0;
}

// A batch without lookups: no sort pass runs that could check the offsets, and the groupings are
// empty (every range of every segment array is [0, 0)).
template <bool BATCHED>
__global__ void k_empty_plan(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  check_offsets(d, u);
  if (u <= d.sh.n3) d.plan.i3_seg[u] = 0;
  if (u <= d.sh.n2) d.plan.i2_seg[u] = 0;
  if (u <= d.sh.n1) d.plan.i1_seg[u] = 0;
}

// ------------------------------------------------------------------ LSD radix pass
#define TT_SORT_MAX_PASSES 4  // 31 key bits in digits of at most 10 bits
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
k_radix_hist(TTArg<BATCHED> a, int which, int in_a, int shift, int bits, int pass) {
  const TTDev &d = a.get();
  const SortBufs sb = sort_bufs(d, which);
  const int ntiles = sb.ntiles;
  if ((int)blockIdx.x >= ntiles) return;  // uniform: this table has fewer tiles than the widest
  const int32_t *__restrict__ keys = in_a ? sb.ka : sb.kb;
  int32_t *__restrict__ hist = d.tmp.hist + pass * ((size_t)1 << TT_SORT_MAX_BITS) * ((size_t)d.sort_tiles + 1);
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
k_radix_binscan(TTArg<BATCHED> a, int which, int nbins, int pass) {
  const TTDev &d = a.get();
  const int ntiles = sort_bufs(d, which).ntiles;
  int32_t *__restrict__ bin_total = d.tmp.bin_total;
  __shared__ int tmp[TT_BLOCK / TT_WAVE + 1];
  int32_t *col = d.tmp.hist + pass * ((size_t)1 << TT_SORT_MAX_BITS) * ((size_t)d.sort_tiles + 1) + blockIdx.x;
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

// Stable scatter.  Wavefront w of a tile owns its keys [w*256, w*256 + 256) and ranks them in four
// rounds of 64 (position order), keeping per-digit running counts in its own row of wave_cnt; one
// scan over the four rows per digit then gives every wavefront its base inside the tile's run of
// that digit.  Equal digits keep their relative order: tiles in order, wavefronts in order, rounds
// in order, lanes in order.
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_radix_scatter(TTArg<BATCHED> a, int which, int in_a, int shift, int bits, int self_scan, int status, int pass,
                int next_bits) {
  const TTDev &d = a.get();
  const SortBufs sb = sort_bufs(d, which);
  const int ntiles = sb.ntiles;
  if (status) {  // first pass of the main sort: this launch also covers the bag offsets
#pragma unroll
    for (int i = 0; i < TT_SORT_ITEMS; ++i) check_offsets(d, blockIdx.x * TT_SORT_TILE + i * TT_BLOCK + threadIdx.x);
  }
  if ((int)blockIdx.x >= ntiles) return;  // uniform
  const int32_t *__restrict__ keys_in = in_a ? sb.ka : sb.kb, *__restrict__ vals_in = in_a ? sb.va : sb.vb;
  int32_t *__restrict__ keys_out = in_a ? sb.kb : sb.ka, *__restrict__ vals_out = in_a ? sb.vb : sb.va;
  // pass p of the main sort reads its own [tile][bin] array; with next_bits > 0 it also counts, per
  // destination tile, the digits of the next pass (integer atomics: the counts do not depend on the
  // order), so that the next pass needs no histogram launch
  const size_t hist_stride = ((size_t)1 << TT_SORT_MAX_BITS) * ((size_t)d.sort_tiles + 1);
  const int32_t *__restrict__ count_ptr = sb.count_ptr, *__restrict__ hist = d.tmp.hist + pass * hist_stride,
                *__restrict__ bin_total = d.tmp.bin_total;
  int32_t *hist_next = d.tmp.hist + (pass + 1) * hist_stride;
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
    if (status && pos < count && keys_r[i] == d.sh.sentinel) atomicOr(&d.plan.counts[4], 1);  // an index was out of range
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
  unsigned long long twins[TT_SORT_ITEMS];  // lanes of the round with the same digit in this and the next pass
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
    twins[i] = mask;
    for (int b = 0; b < next_bits; ++b) {
      const bool bit = (keys_r[i] >> (shift + bits + b)) & 1;
      unsigned long long m = __ballot(valid && bit);
      twins[i] &= bit ? m : ~m;
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
    const bool valid = pos < count;
    int dst = 0;
    if (valid) {
      dst = gofs[digit[i]] + wave_cnt[wave][digit[i]] + rank[i];
      keys_out[dst] = keys_r[i];
      vals_out[dst] = vals_r[i];
    }
    if (next_bits > 0) {  // uniform
      // One addition per group of lanes with the same two digits, made by the group's first lane:
      // the lanes of a group go to places less than 64 apart, hence to one destination tile unless
      // a tile border falls inside the group, and then the lanes behind the border add for themselves.
      // (Lookups of one hot row would otherwise all add to one address, one after the other.)
      const int dtile = dst / TT_SORT_TILE;
      const int first = valid ? __ffsll(twins[i]) - 1 : lane;
      const int dtile_first = __shfl(dtile, first);
      const unsigned long long apart = __ballot(valid && dtile != dtile_first);
      const int n = dtile != dtile_first ? 1 : lane == first ? __popcll(twins[i] & ~apart) : 0;
      if (valid && n > 0)
        atomicAdd(hist_next + (size_t)dtile * (1 << next_bits) + ((keys_r[i] >> (shift + bits)) & ((1 << next_bits) - 1)), n);
    }
  }
}

// ------------------------------------------------------------------ distinct rows / prefixes
#define TT_UNIQ_ITEMS 4
#define TT_UNIQ_TILE (TT_BLOCK * TT_UNIQ_ITEMS)
#define TT_UNIQ_SELF_SCAN_TILES 1024  // up to this many tiles k_uniq_emit does without k_uniq_scan
#define TT_GROUP_MAX_TILES 512        // up to this many tiles of (capacity for) distinct rows the groupings take one launch

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
// group_keys = 0: the groupings take their keys from uniq_row / uniq_pref (k_group), nothing is
// emitted for them here.  (Counting the heads of the earlier tiles from the keys themselves inside
// this kernel, instead of a k_uniq_reduce launch, was measured: the last tile's workgroup then reads
// the whole key array and the kernel takes 35 us instead of 4.5 + 9.5.)
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_uniq_emit(TTArg<BATCHED> a, int a3, int a2, int self_scan, int group_keys) {
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
      if (group_keys) {
        k3[slot_r] = key % n3;
        v3[slot_r] = slot_r;
      }
    }
    if (hp[i]) {
      uniq_pref[ep - 1] = key / n3;
      pref_seg[ep - 1] = slot_r;
      if (group_keys) {
        k2[ep - 1] = (key / n3) % n2;
        v2[ep - 1] = ep - 1;
      }
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

// ------------------------------------------------------------------ groupings in one launch
// Stable single-pass counting sort of `count` items by a key below 2^bits (bits <= 10): this
// workgroup places the items of tile `tile`.  key_of(src[pos]) is the key of item pos, place(dst, pos,
// key) stores it at its sorted position, seg(bin, start) receives -- from tile 0 -- the start of
// every bin's run (= the number of items with a smaller key).  No histogram launch: every workgroup
// counts all keys itself (per bin: in total, and before its tile), which for the few thousand
// distinct rows / prefixes of a batch is cheaper than a second launch.
struct CountingSortLds {
  int gofs[1 << TT_SORT_MAX_BITS];  // bin totals, then global offset of (bin, this tile)
  int pre[1 << TT_SORT_MAX_BITS];   // per bin: items before this tile
  int wave_cnt[TT_BLOCK / TT_WAVE][1 << TT_SORT_MAX_BITS];
  int tmp[TT_BLOCK / TT_WAVE + 1];
};
template <class KeyOf, class Place, class Seg>
__device__ __forceinline__ void counting_sort_tile(CountingSortLds &L, const int32_t *__restrict__ src, int count,
                                                   int bits, int tile, KeyOf key_of, Place place, Seg seg) {
  constexpr int MAXB = 1 << TT_SORT_MAX_BITS;
  constexpr int NW = TT_BLOCK / TT_WAVE;
  constexpr int PER = MAXB / TT_BLOCK;
  int *gofs = L.gofs, *pre = L.pre, *tmp = L.tmp;
  int (*wave_cnt)[MAXB] = L.wave_cnt;
  const int nbins = 1 << bits, base = tile * TT_SORT_TILE;
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;
  // uniform: the launch is sized by the capacity; a tile past the actual count has nothing to place
  // (tile 0 still writes the segment starts)
  if (base >= count && tile != 0) return;
  for (int b = threadIdx.x; b < nbins; b += TT_BLOCK) { gofs[b] = 0; pre[b] = 0; }
  __syncthreads();
  {  // eight loads in flight per thread (src is 16-byte aligned: four items per load)
    constexpr int INFLIGHT = 8;
    for (int p4 = threadIdx.x * 4; p4 < count; p4 += TT_BLOCK * 4 * INFLIGHT) {
      int4 v[INFLIGHT];
#pragma unroll
      for (int j = 0; j < INFLIGHT; ++j) {
        const int at = p4 + j * TT_BLOCK * 4;
        v[j] = at < count ? *reinterpret_cast<const int4 *>(src + at) : make_int4(0, 0, 0, 0);  // (the arrays are padded past `count`)
      }
#pragma unroll
      for (int j = 0; j < INFLIGHT; ++j) {
        const int at = p4 + j * TT_BLOCK * 4;
        const int vv[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (at + i < count) {
            const int k = key_of(vv[i]);
            atomicAdd(&gofs[k], 1);
            if (at + i < base) atomicAdd(&pre[k], 1);
          }
      }
    }
  }
  __syncthreads();
  {
    int loc[PER], sum = 0;
    const int b0 = threadIdx.x * PER;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      loc[k] = b0 + k < nbins ? gofs[b0 + k] : 0;
      sum += loc[k];
    }
    int total, ex = tt_block_excl_scan(sum, tmp, &total);  // (two barriers: every thread has read its totals)
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      if (b0 + k < nbins) {
        if (tile == 0) seg(b0 + k, ex);
        gofs[b0 + k] = ex + pre[b0 + k];
#pragma unroll
        for (int w = 0; w < NW; ++w) wave_cnt[w][b0 + k] = 0;
      }
      ex += loc[k];
    }
  }
  __syncthreads();
  if (base >= count) return;  // uniform
  int keys_r[TT_SORT_ITEMS], rank[TT_SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < TT_SORT_ITEMS; ++i) {  // wavefront w ranks its contiguous 256 items in four rounds of 64
    const int pos = base + (wave * TT_SORT_ITEMS + i) * TT_WAVE + lane;
    const bool valid = pos < count;
    keys_r[i] = valid ? key_of(src[pos]) : 0;
    unsigned long long mask = __ballot(valid);  // lanes of this round with the same key
    for (int b = 0; b < bits; ++b) {
      const bool bit = (keys_r[i] >> b) & 1;
      unsigned long long m = __ballot(valid && bit);
      mask &= bit ? m : ~m;
    }
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (TT_WAVE - lane));
    const int rank_in_round = __popcll(mask & lt);
    const int prev = valid ? wave_cnt[wave][keys_r[i]] : 0;  // this wavefront's earlier rounds
    tt_wave_lds_order();
    if (valid && rank_in_round == 0) wave_cnt[wave][keys_r[i]] = prev + __popcll(mask);
    tt_wave_lds_order();
    rank[i] = prev + rank_in_round;
  }
  __syncthreads();
  {  // per key: counts of the wavefronts -> their bases inside the tile's run of the key
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
    if (pos < count) place(gofs[keys_r[i]] + wave_cnt[wave][keys_r[i]] + rank[i], pos, keys_r[i]);
  }
}

// The three groupings of a plan in ONE launch (tables whose factors are below 1024):
//   workgroups [0, nb3):        distinct rows stably sorted by i3 -> rows_by_i3, i3_of_sorted, i3_seg
//   workgroups [nb3, nb3+nb2):  distinct prefixes stably sorted by i2 -> prefs_by_i2, i2_seg, and the
//                               packed per-prefix records the matrix-core kernels read (pref_meta)
//   last workgroup:             i1_seg (prefix slots are already in i1 order: a histogram suffices)
// Each role is its own code path with its own buffers (no buffer is chosen from the workgroup index).
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_group(TTArg<BATCHED> a, int nb3, int nb2, int bits3, int bits2, int bits1) {
  const TTDev &d = a.get();
  const int32_t *__restrict__ counts = d.plan.counts;
  const int ur = counts[0], up = counts[1];
  const int n1 = d.sh.n1, n2 = d.sh.n2, n3 = d.sh.n3;
  const unsigned mul3 = d.sh.mul3, sh3 = d.sh.sh3, mul2 = d.sh.mul2, sh2 = d.sh.sh2;
  __shared__ CountingSortLds L;
  if ((int)blockIdx.x < nb3) {
    const int32_t *__restrict__ uniq_row = d.plan.uniq_row;
    int32_t *__restrict__ rows_by_i3 = d.plan.rows_by_i3, *__restrict__ i3_of_sorted = d.plan.i3_of_sorted,
            *__restrict__ i3_seg = d.plan.i3_seg;
    counting_sort_tile(L, uniq_row, ur, bits3, blockIdx.x,
                       [&](int row) { return row - tt_div(row, mul3, sh3) * n3; },
                       [&](int dst, int pos, int key) { rows_by_i3[dst] = pos; i3_of_sorted[dst] = key; },
                       [&](int bin, int start) { if (bin <= n3) i3_seg[bin] = start; });
  } else if ((int)blockIdx.x < nb3 + nb2) {
    const int32_t *__restrict__ uniq_pref = d.plan.uniq_pref, *__restrict__ pref_seg = d.plan.pref_seg;
    int32_t *__restrict__ prefs_by_i2 = d.plan.prefs_by_i2, *__restrict__ i2_seg = d.plan.i2_seg;
    int4 *__restrict__ pref_meta = reinterpret_cast<int4 *>(d.plan.pref_meta);
    counting_sort_tile(L, uniq_pref, up, bits2, blockIdx.x - nb3,
                       [&](int pref) { return pref - tt_div(pref, mul2, sh2) * n2; },
                       [&](int dst, int pos, int) {
                         prefs_by_i2[dst] = pos;
                         const int u0 = pref_seg[pos];  // i1, first distinct-row slot, distinct rows, prefix slot
                         pref_meta[dst] = make_int4(tt_div(uniq_pref[pos], mul2, sh2), u0, pref_seg[pos + 1] - u0, pos);
                       },
                       [&](int bin, int start) { if (bin <= n2) i2_seg[bin] = start; });
  } else {
    const int32_t *__restrict__ uniq_pref = d.plan.uniq_pref;
    int32_t *__restrict__ i1_seg = d.plan.i1_seg;
    // a counting sort whose items stay where they are: only the bin starts are kept
    counting_sort_tile(L, uniq_pref, up, bits1, 0, [&](int pref) { return tt_div(pref, mul2, sh2); }, [&](int, int, int) {},
                       [&](int bin, int start) { if (bin <= n1) i1_seg[bin] = start; });
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
// `status_tiles` > 0 marks the main sort: its first pass finds its histogram already there (the
// kernel that extracted the keys counted the first digit) and its first scatter launch is made wide
// enough to check the bag offsets as well.
tt_status radix_sort(const TTBatch &b, int which, int max_tiles, int key_bits, hipStream_t s, int status_tiles) {
  const RadixPlan rp = radix_plan(key_bits);
  if (max_tiles == 0) return TT_OK;
  int in_a = (rp.passes % 2) == 0;
  int shift = 0;
  for (int p = 0; p < rp.passes; ++p) {
    const int bits = (key_bits - shift) < rp.bits_per_pass ? (key_bits - shift) : rp.bits_per_pass;
    const int self_scan = max_tiles <= TT_SELF_SCAN_TILES ? 1 : 0;
    const bool main_sort = status_tiles > 0;
    const int status = (main_sort && p == 0) ? 1 : 0;
    // The main sort finds the histogram of pass 0 already there (counted while the keys were extracted).
    // Short main sorts, whose cost is launches, also let the scatter of pass p count pass p + 1 (atomic
    // additions per destination tile); long ones keep the histogram launch, which is cheaper than the
    // atomics from a few hundred tiles on (335 k keys: 4.4 us against 13 us more per scatter).
    const bool count_next = main_sort && max_tiles <= TT_SELF_SCAN_TILES;
    const int pass = main_sort ? p : 0;
    int next_bits = 0;
    if (count_next && p + 1 < rp.passes) {
      const int left = key_bits - shift - bits;
      next_bits = left < rp.bits_per_pass ? left : rp.bits_per_pass;
    }
    if (!main_sort || (p > 0 && !count_next))
      TT_LAUNCH(k_radix_hist, max_tiles, TT_BLOCK, 0, s, b, which, in_a, shift, bits, pass);
    if (!self_scan) TT_LAUNCH(k_radix_binscan, 1 << bits, TT_BLOCK, 0, s, b, which, 1 << bits, pass);
    {
      TTProfScope prof(which == 0 ? &b.host[0].plan : nullptr, TT_KERNEL_SORT_SCATTER, s);
      const int grid = status && status_tiles > max_tiles ? status_tiles : max_tiles;
      TT_LAUNCH(k_radix_scatter, grid, TT_BLOCK, 0, s, b, which, in_a, shift, bits, self_scan, status, pass, next_bits);
    }
    shift += bits;
    in_a = !in_a;
  }
  return tt_launch_status();
}

}  // namespace

int ttk_radix_passes(int key_bits) { return radix_plan(key_bits).passes; }

tt_status ttk_sort_slot1(const TTDev &d, int key_bits, hipStream_t s) {
  const TTBatch b = {1, &d, nullptr};
  return radix_sort(b, 1, tt_ceil_div(d.plan.max_rows, TT_SORT_TILE), key_bits, s, 0);
}

size_t tt_sort_tmp_bytes(int64_t nnz, int64_t max_rows, int64_t max_prefixes) {
  const size_t ntiles = (size_t)tt_ceil_div(nnz, TT_SORT_TILE) + 1;
  const size_t utiles = (size_t)tt_ceil_div(nnz, TT_UNIQ_TILE) + 1;
  size_t ints = 3 * (size_t)nnz + 2 * (size_t)max_rows + 3 * (size_t)max_prefixes +
                TT_SORT_MAX_PASSES * ((size_t)1 << TT_SORT_MAX_BITS) * ntiles + ((size_t)1 << TT_SORT_MAX_BITS) +
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
  t.hist = take(TT_SORT_MAX_PASSES * ((size_t)1 << TT_SORT_MAX_BITS) * ntiles);  // one [tile][bin] array per pass
  t.bin_total = take((size_t)1 << TT_SORT_MAX_BITS);
  t.tile_sums = take(2 * ((size_t)tt_ceil_div(plan->nnz, TT_UNIQ_TILE) + 1));
  return t;
}

tt_status ttk_reorder(const TTBatch &b, hipStream_t s) {
  // main sort: keys in [0, sentinel]
  const int key_bits = bit_length(tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.sentinel; }));
  const RadixPlan rp0 = radix_plan(key_bits);
  const int in_a = (rp0.passes % 2) == 0;
  const int bits0 = key_bits < rp0.bits_per_pass ? key_bits : rp0.bits_per_pass;
  const int tiles0 = (int)tt_batch_max(b, [](const TTDev &d) { return (long long)d.sort_tiles; });
  // first kernel: counters, keys, bags, histogram of the first digit
  TT_LAUNCH(k_extract_keys, tiles0 > 0 ? tiles0 : 1, TT_BLOCK, 0, s, b, in_a, bits0, rp0.passes);
  // the first scatter pass also checks the bag offsets (one thread per offset)
  const long long bags1 = tt_batch_max(b, [](const TTDev &d) { return (long long)d.num_bags + 1; });
  if (tiles0 == 0) {
    const long long cover = tt_batch_max(b, [](const TTDev &d) {
      long long m = d.sh.n1 > d.sh.n2 ? d.sh.n1 : d.sh.n2;
      m = (m > d.sh.n3 ? m : (long long)d.sh.n3) + 1;
      return m > d.num_bags + 1 ? m : (long long)d.num_bags + 1; });
    TT_LAUNCH(k_empty_plan, tt_ceil_div(cover, TT_BLOCK), TT_BLOCK, 0, s, b);
    return tt_launch_status();  // no lookups: the first kernel has left an empty plan
  }
  tt_status st = radix_sort(b, 0, tiles0, key_bits, s, tt_ceil_div(bags1, TT_SORT_TILE));
  if (st != TT_OK) return st;

  // distinct rows and prefixes
  const int utiles = (int)tt_batch_max(b, [](const TTDev &d) {
    return (long long)tt_ceil_div(d.nnz, TT_UNIQ_TILE); });
  // groupings: distinct rows by i3, distinct prefixes by i2 (stable), i1 ranges
  const long long n1max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n1; });
  const long long n2max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n2; });
  const long long n3max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n3; });
  // (the values n3, n2, n1 themselves get a bin: its start is the item count)
  const int bits3 = bit_length(n3max), bits2 = bit_length(n2max), bits1 = bit_length(n1max);
  const long long max_rows = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_rows; });
  const long long max_pref = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_prefixes; });
  const int nb3 = tt_ceil_div(max_rows, TT_SORT_TILE), nb2 = tt_ceil_div(max_pref, TT_SORT_TILE);
  // one launch for all three groupings when every key fits one radix digit and the inputs are short
  // enough that every workgroup can count all keys itself
  const bool grouped = bits3 <= TT_SORT_MAX_BITS && bits2 <= TT_SORT_MAX_BITS && bits1 <= TT_SORT_MAX_BITS &&
                       nb3 <= TT_GROUP_MAX_TILES;
  const int sb3 = bit_length(n3max - 1), sb2 = bit_length(n2max - 1);  // key widths of the separate grouping sorts
  const int a3 = (radix_plan(sb3).passes % 2) == 0, a2 = (radix_plan(sb2).passes % 2) == 0;
  // short inputs: every emit workgroup adds up the earlier tiles' sums itself (no scan launch)
  const int uniq_mode = utiles <= TT_UNIQ_SELF_SCAN_TILES ? 1 : 0;
  TT_LAUNCH(k_uniq_reduce, utiles, TT_BLOCK, 0, s, b);
  if (uniq_mode == 0) TT_LAUNCH(k_uniq_scan, 1, TT_BLOCK, 0, s, b);
  TT_LAUNCH(k_uniq_emit, utiles, TT_BLOCK, 0, s, b, a3, a2, uniq_mode, grouped ? 0 : 1);
  if (grouped) {
    TT_LAUNCH(k_group, nb3 + nb2 + 1, TT_BLOCK, 0, s, b, nb3, nb2, bits3, bits2, bits1);
    return tt_launch_status();
  }
  st = radix_sort(b, 1, nb3, sb3, s, 0);
  if (st != TT_OK) return st;
  st = radix_sort(b, 2, nb2, sb2, s, 0);
  if (st != TT_OK) return st;
  // one thread per sorted position (and at least one per segment boundary when a count is zero)
  const long long nmax = tt_batch_max(b, [](const TTDev &d) {
    long long m = d.sh.n1 > d.sh.n2 ? d.sh.n1 : d.sh.n2;
    m = m > d.sh.n3 ? m : (long long)d.sh.n3;
    m += 1;
    return m > d.plan.max_rows ? m : (long long)d.plan.max_rows; });
  TT_LAUNCH(k_seg_bounds, tt_ceil_div(nmax, TT_BLOCK), TT_BLOCK, 0, s, b);
  return tt_launch_status();
}
