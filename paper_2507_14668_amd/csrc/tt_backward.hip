// Backward pass of the TT embedding bag (paper Section III-D backward equation, Section III-E
// in-advance gradient aggregation) and the gradient-descent core update.
//
// Planned arm:
//   1. merge grad_out over all occurrences of each distinct row (segmented gather-sum);
//   2. per distinct prefix: rebuild P12, and for each distinct row under it form the core-2
//      contribution P12^T g and accumulate the right partial H = sum_rows g G3[i3]^T;
//      then the core-0 contribution H G2[i2]^T;
//   3. reduce the per-row / per-prefix contributions into core-shaped gradients with sorted
//      segmented sums (core 2 by i3, core 0 by i1) and a per-i2 accumulation (core 1).
//   No floating-point atomics: every output element is written once, in a fixed order.
// Naive arm: one workgroup per lookup, full chain, atomicAdd into the core gradients.
#include "tt_internal.h"

namespace {

// ------------------------------------------------------------------ two-stage segmented sum
// Positions 0..M-1 carry a vector src[gidx[pos]][W] and a non-decreasing segment id
// seg_src[pos]/seg_div; seg_off[s]..seg_off[s+1] is the position range of segment s.
// Stage 1 walks fixed chunks of `chunk` positions in order; a segment that lies inside one
// chunk is finished there, otherwise the chunk leaves a partial: slot 0 = run that began before
// the chunk, slot 1 = run that begins in the chunk and continues past its end.
// A position may carry `nsub` consecutive vectors (src[(gidx[pos]*nsub + t)][W], t < nsub),
// which are added in order first.
// Output element e of segment s goes to out[((e/out_inner)*nseg + s)*out_inner + e%out_inner]
// (out_inner = W gives a contiguous [nseg][W] array; out_inner = d3 gives core-2 layout).
template <int VEC>
struct Vec {
  float v[VEC];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] = 0.f;
  }
  __device__ __forceinline__ void load(const float *p) {
    if (VEC == 4) {
      const float4 t = *reinterpret_cast<const float4 *>(p);
      v[0] = t.x; v[1 % VEC] = t.y; v[2 % VEC] = t.z; v[3 % VEC] = t.w;
    } else {
      v[0] = *p;
    }
  }
  __device__ __forceinline__ void load_stream(const float *p) {  // data read exactly once
    if (VEC == 4) {
      const float4 t = tt_load_stream4(p);
      v[0] = t.x; v[1 % VEC] = t.y; v[2 % VEC] = t.z; v[3 % VEC] = t.w;
    } else {
      v[0] = *p;
    }
  }
  __device__ __forceinline__ void store(float *p) const {
    if (VEC == 4) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1 % VEC], v[2 % VEC], v[3 % VEC]);
    else *p = v[0];
  }
  // p <- p - lr * v   (the fused core update: the finished gradient slice is never stored)
  __device__ __forceinline__ void store_sgd(float *p, float lr) const {
    Vec old;
    old.load(p);
#pragma unroll
    for (int k = 0; k < VEC; ++k) old.v[k] = fmaf(-lr, v[k], old.v[k]);
    old.store(p);
  }
  __device__ __forceinline__ void add(const Vec &o) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] += o.v[k];
  }
};

__device__ __forceinline__ size_t seg_out_index(int s, int e, int out_inner, int nseg) {
  const int hi = e / out_inner, lo = e - hi * out_inner;
  return ((size_t)hi * nseg + s) * out_inner + lo;
}

// The three segmented sums of the backward pass, described per table on the device.
enum { SEG_GAGG = 0, SEG_DG3 = 1, SEG_DG1 = 2 };
struct SegView {
  int W;                     // vector width
  const int32_t *count_ptr;  // device: number of positions
  const int32_t *seg_src;
  int seg_div;
  const int32_t *gidx;
  const int32_t *seg_off;
  const float *src;
  int nsub;                  // vectors per position
  float *out;
  int out_inner;
  int nseg;                  // number of segments (output layout / dense zero fill)
  int dense;
  float *partial;
  int fused;                 // out is the core itself: finished sums are applied as out -= lr * sum
  float lr;
  int stream_src;            // every source vector is read once: non-temporal loads
};
__device__ __forceinline__ SegView seg_view(const TTDev &d, int kind) {
  SegView v;
  v.partial = d.plan.partial;
  v.fused = 0; v.lr = d.lr;
  v.stream_src = 1;  // the hand-off buffers are read once; the output gradients only with one lookup per bag
  if (kind == SEG_GAGG) {  // merge grad_out over the occurrences of each distinct row
    v.W = d.sh.D; v.count_ptr = d.plan.counts + 2; v.seg_src = d.plan.slot_of_sorted; v.seg_div = 1;
    v.gidx = d.plan.bag_of_sorted; v.seg_off = d.plan.row_seg; v.src = d.grad_out; v.nsub = 1;
    v.out = d.plan.gagg; v.out_inner = d.sh.D; v.nseg = (int)d.plan.max_rows; v.dense = 0;
    v.stream_src = d.nnz == d.num_bags;
  } else if (kind == SEG_DG3) {  // core 2: per-row contributions of all rows sharing i3
    v.W = d.sh.S3; v.count_ptr = d.plan.counts + 0; v.seg_src = d.plan.i3_of_sorted; v.seg_div = 1;
    v.gidx = d.plan.rows_by_i3; v.seg_off = d.plan.i3_seg; v.src = d.plan.t3buf; v.nsub = 1;
    v.out = d.dg[2]; v.out_inner = d.sh.d3; v.nseg = d.sh.n3; v.dense = 1;
    if (d.fused) { v.out = const_cast<float *>(d.g[2]); v.dense = 0; v.fused = 1; }
  } else {  // core 0: per-prefix contributions of all prefixes sharing i1 (contiguous)
    v.W = d.sh.S1; v.count_ptr = d.plan.counts + 1; v.seg_src = d.plan.uniq_pref; v.seg_div = d.sh.n2;
    v.gidx = nullptr; v.seg_off = d.plan.i1_seg; v.src = d.plan.t1buf; v.nsub = d.strips;
    v.out = d.dg[0]; v.out_inner = d.sh.S1; v.nseg = d.sh.n1; v.dense = 1;
    if (d.fused) { v.out = const_cast<float *>(d.g[0]); v.dense = 0; v.fused = 1; }
  }
  return v;
}

// One launch serves one segmented sum, or two of the same vector width side by side (the first
// `blocks` workgroups the first kind, the rest the second, whose partials follow the first kind's
// in the table's partial buffer).
struct SegLaunch {
  int kind, chunk, blocks;
  int kind_b, chunk_b;  // kind_b < 0: a single sum
};
struct SegPick { int kind, chunk, bid, nblk; size_t poff; };
__device__ __forceinline__ SegPick seg_pick(const SegLaunch &L, const TTDev &d) {
  SegPick p = {L.kind, L.chunk, (int)blockIdx.x, L.kind_b < 0 ? (int)gridDim.x : L.blocks, 0};
  if (L.kind_b >= 0 && (int)blockIdx.x >= L.blocks) {
    p.kind = L.kind_b; p.chunk = L.chunk_b; p.bid = (int)blockIdx.x - L.blocks;
    p.nblk = (int)gridDim.x - L.blocks;
    // the first kind's share of this table's partial buffer: two slots per chunk it can have
    const long long cap = L.kind == SEG_GAGG ? d.plan.nnz : (L.kind == SEG_DG3 ? d.plan.max_rows : d.plan.max_prefixes);
    const int W = L.kind == SEG_GAGG ? d.sh.D : (L.kind == SEG_DG3 ? d.sh.S3 : d.sh.S1);
    p.poff = (size_t)((cap + L.chunk - 1) / L.chunk + 1) * 2 * W;
  }
  return p;
}

template <bool BATCHED, int VEC>
__global__ void __launch_bounds__(TT_BLOCK)
k_seg_stage1(TTArg<BATCHED> arg, SegLaunch L, int lanes) {
  const SegPick pk = seg_pick(L, arg.get());
  const int chunk = pk.chunk;
  const SegView sv = seg_view(arg.get(), pk.kind);
  const int W = sv.W, seg_div = sv.seg_div, nsub = sv.nsub, out_inner = sv.out_inner, nseg = sv.nseg;
  const int32_t *__restrict__ seg_src = sv.seg_src, *__restrict__ gidx = sv.gidx;
  const float *__restrict__ src = sv.src;
  float *__restrict__ out = sv.out, *__restrict__ partial = sv.partial + pk.poff;
  const int M = *sv.count_ptr;
  const int nchunks = (M + chunk - 1) / chunk;
  const int fused = sv.fused, stream_src = sv.stream_src;
  const float lr = sv.lr;
  const int groups = blockDim.x / lanes, g = threadIdx.x / lanes, lane = threadIdx.x - g * lanes;
  extern __shared__ float red[];  // [groups][W]
  for (int c = pk.bid * groups + g; c < nchunks; c += pk.nblk * groups) {
    const int lo = c * chunk, hi = lo + chunk, end = hi < M ? hi : M;
    // the `groups` chunks of this workgroup; a segment that starts before and ends after them makes
    // every lane group see the same thing, so `merged` is uniform over the workgroup
    const int block_lo = (c - g) * chunk, block_hi = block_lo + groups * chunk;
    bool merged = false;
    // segment ids just outside the chunk and just outside the workgroup's range (-1 / -2: nothing there)
    const int s_before = lo > 0 ? seg_src[lo - 1] / seg_div : -1;
    const int s_after = hi < M ? seg_src[hi] / seg_div : -2;
    const int s_blk_before = block_lo > 0 ? seg_src[block_lo - 1] / seg_div : -1;
    const int s_blk_after = block_hi < M ? seg_src[block_hi] / seg_div : -2;
    // Where a finished run goes is decided from the segment ids next to the chunk and next to the
    // workgroup's range (ids are non-decreasing), not from the segment's offsets: those would be two
    // dependent loads at every segment change.  `at_end`: the run reaches the chunk's last position.
    // `active`: this lane holds columns of the vector (the flag `merged` is set by idle lanes too: it
    // decides a workgroup barrier).
    auto flush = [&](const Vec<VEC> &acc, int cur, int e, bool active, bool at_end) {
      const bool starts_in = cur != s_before;          // the segment begins inside the chunk
      const bool ends_in = !at_end || cur != s_after;  // ... and ends inside it
      if (starts_in && ends_in) {
        if (active) {
          float *dst = out + seg_out_index(cur, e, out_inner, nseg);
          if (fused) acc.store_sgd(dst, lr); else acc.store(dst);
        }
      } else if (cur == s_blk_before && cur == s_blk_after) {  // it covers the workgroup's whole range:
        if (active) acc.store(red + (size_t)g * W + e);       // one partial for the workgroup, summed below
        merged = true;
      } else if (active) acc.store(partial + ((size_t)c * 2 + (starts_in ? 1 : 0)) * W + e);
    };
    auto load_row = [&](int row, int e, Vec<VEC> &x) {
      if (stream_src) x.load_stream(src + (size_t)row * nsub * W + e);
      else x.load(src + (size_t)row * nsub * W + e);
      for (int t = 1; t < nsub; ++t) {
        Vec<VEC> y;
        y.load(src + ((size_t)row * nsub + t) * W + e);
        x.add(y);
      }
    };
    if (lanes >= TT_SEG_UNROLL) {
      // The lanes of the group fetch the segment ids and gather indices of `lanes` positions at once,
      // one position per lane, and hand them round with lane shuffles: one round trip for the indices
      // of a whole block of positions instead of one in front of every group of gathers.  (Every lane
      // runs every shuffle; positions past the chunk's end carry the id -3 and are skipped.)
      for (int e0 = 0; e0 < W; e0 += lanes * VEC) {
        const int e = e0 + lane * VEC;
        const bool active = e < W;
        Vec<VEC> acc;
        acc.zero();
        int cur = -1;
        for (int sub = lo; sub < hi; sub += lanes) {
          const int mine = sub + lane;
          int my_sg = -3, my_row = 0;
          if (mine < end) {
            my_sg = seg_src[mine] / seg_div;
            my_row = gidx ? gidx[mine] : mine;
          }
          const int cnt = (hi - sub) < lanes ? (hi - sub) : lanes;  // a multiple of TT_SEG_UNROLL
          for (int k = 0; k < cnt; k += TT_SEG_UNROLL) {
            int sg[TT_SEG_UNROLL];
            Vec<VEC> x[TT_SEG_UNROLL];
#pragma unroll
            for (int u = 0; u < TT_SEG_UNROLL; ++u) {
              sg[u] = __shfl(my_sg, k + u, lanes);
              const int row = __shfl(my_row, k + u, lanes);
              if (sg[u] != -3 && active) load_row(row, e, x[u]); else x[u].zero();
            }
#pragma unroll
            for (int u = 0; u < TT_SEG_UNROLL; ++u) {
              if (sg[u] == -3) continue;
              if (sg[u] != cur) {
                if (cur >= 0) flush(acc, cur, e, active, false);
                cur = sg[u];
                acc.zero();
              }
              acc.add(x[u]);
            }
          }
        }
        if (cur >= 0) flush(acc, cur, e, active, true);
      }
    } else {
      for (int e = lane * VEC; e < W; e += lanes * VEC) {
        Vec<VEC> acc;
        acc.zero();
        int cur = -1;
        for (int pos = lo; pos < end; ++pos) {
          const int sgk = seg_src[pos] / seg_div;
          Vec<VEC> x;
          load_row(gidx ? gidx[pos] : pos, e, x);
          if (sgk != cur) {
            if (cur >= 0) flush(acc, cur, e, true, false);
            cur = sgk;
            acc.zero();
          }
          acc.add(x);
        }
        if (cur >= 0) flush(acc, cur, e, true, true);
      }
    }
    if (merged) {  // uniform: the chunks' sums in chunk order -> slot 0 of the workgroup's first chunk
      __syncthreads();
      if (g == 0)
        for (int e = lane * VEC; e < W; e += lanes * VEC) {
          Vec<VEC> acc, x;
          acc.load(red + e);
          for (int k = 1; k < groups; ++k) {
            x.load(red + (size_t)k * W + e);
            acc.add(x);
          }
          acc.store(partial + ((size_t)(c - g) * 2) * W + e);
        }
      __syncthreads();
    }
  }
}

#ifndef TT_SEG2_UNROLL
#define TT_SEG2_UNROLL 8  // partials a lane group of stage 2 keeps in flight
#endif
// Stage 2: workgroup per chunk.  The chunk in which a multi-chunk segment begins owns it and adds
// its own slot-1 partial and the slot-0 partials of the following chunks, in chunk order.
// With `dense`, workgroup c also zero-fills segment c if it is empty.
// LDS: red[groups][W]
template <bool BATCHED, int VEC>
__global__ void __launch_bounds__(TT_BLOCK)
k_seg_stage2(TTArg<BATCHED> arg, SegLaunch L, int lanes) {
  const SegPick pk = seg_pick(L, arg.get());
  const int chunk = pk.chunk;
  const SegView sv = seg_view(arg.get(), pk.kind);
  const int W = sv.W, seg_div = sv.seg_div, out_inner = sv.out_inner, nseg = sv.nseg, dense = sv.dense;
  const int32_t *__restrict__ seg_src = sv.seg_src, *__restrict__ seg_off = sv.seg_off;
  float *__restrict__ out = sv.out;
  const float *__restrict__ partial = sv.partial + pk.poff;
  extern __shared__ float red[];
  const int M = *sv.count_ptr;
  const int nchunks = (M + chunk - 1) / chunk;
  const int c = pk.bid;
  const int groups = blockDim.x / lanes, g = threadIdx.x / lanes, lane = threadIdx.x - g * lanes;
  if (dense && c < nseg && seg_off[c] == seg_off[c + 1] && g == 0) {
    Vec<VEC> z;
    z.zero();
    for (int e = lane * VEC; e < W; e += lanes * VEC)
      z.store(out + seg_out_index(c, e, out_inner, nseg));
  }
  if (c >= nchunks) return;  // uniform
  const int lo = c * chunk, hi = lo + chunk, end = hi < M ? hi : M;
  const int s = seg_src[end - 1] / seg_div;
  const int a = seg_off[s], b = seg_off[s + 1];
  if (!(a >= lo && b > hi)) return;  // uniform: no segment starts here and runs past the chunk
  const int c1 = (b - 1) / chunk;
  // Partials to add: slot 0 of the chunks c+1 .. c1, except that stage 1 has left ONE partial (in
  // the first chunk) for every run of `groups` chunks handled by one workgroup that lies strictly
  // inside the segment: the runs B0 .. B1.  Units in order: single chunks before the runs, one per
  // run, single chunks after.
  const int gc = groups * chunk;
  int B0 = a / gc + 1, B1 = (b + gc - 1) / gc - 2;
  int nh = c1 - c, nm = 0, nt = 0;
  if (B0 <= B1) {
    nh = B0 * groups - (c + 1);
    nm = B1 - B0 + 1;
    nt = c1 - (B1 + 1) * groups + 1;
  }
  const int units = nh + nm + nt;
  auto unit_chunk = [&](int u) {
    return u < nh ? c + 1 + u : (u < nh + nm ? (B0 + (u - nh)) * groups : (B1 + 1) * groups + (u - nh - nm));
  };
  for (int e = lane * VEC; e < W; e += lanes * VEC) {
    Vec<VEC> acc;
    acc.zero();
    int u = g;
    for (; u + (TT_SEG2_UNROLL - 1) * groups < units; u += TT_SEG2_UNROLL * groups) {
      Vec<VEC> x[TT_SEG2_UNROLL];  // independent loads in flight, added in unit order
#pragma unroll
      for (int k = 0; k < TT_SEG2_UNROLL; ++k) x[k].load(partial + ((size_t)unit_chunk(u + k * groups) * 2) * W + e);
#pragma unroll
      for (int k = 0; k < TT_SEG2_UNROLL; ++k) acc.add(x[k]);
    }
    for (; u < units; u += groups) {
      Vec<VEC> x;
      x.load(partial + ((size_t)unit_chunk(u) * 2) * W + e);
      acc.add(x);
    }
    acc.store(red + (size_t)g * W + e);
  }
  __syncthreads();
  if (g == 0) {
    for (int e = lane * VEC; e < W; e += lanes * VEC) {
      Vec<VEC> acc, x;
      acc.load(partial + ((size_t)c * 2 + 1) * W + e);
      for (int k = 0; k < groups; ++k) {
        x.load(red + (size_t)k * W + e);
        acc.add(x);
      }
      float *dst = out + seg_out_index(s, e, out_inner, nseg);
      if (sv.fused) acc.store_sgd(dst, sv.lr); else acc.store(dst);
    }
  }
}

// Stage-1 chunk length for `count` positions.  Short chunks give stage 1 more lane groups to hide
// the gather latency with (65 k positions: 8 beats 32 by 2x); long chunks leave stage 2 fewer
// partials to fold for the hottest segment (335 k positions with one segment of 60 k: 32 beats 8).
static int seg_chunk_for(long long count) {
  int c = TT_SEG_MIN_CHUNK;
  while (c < TT_SEG_MAX_CHUNK && (long long)c * 2 * 8192 <= count) c *= 2;
  return c;
}

// Launch shape of one segmented sum over every table of the batch (chunk <= 0: chosen from the count).
struct SegParams { int W, vec, lanes, groups, chunk, nchunks, blocks1; long long blocks2; };
static SegParams seg_params(const TTBatch &b, int kind, int chunk) {
  const TTShape &sh = b.host[0].sh;
  SegParams p;
  p.W = kind == SEG_GAGG ? sh.D : (kind == SEG_DG3 ? sh.S3 : sh.S1);
  const int out_inner = kind == SEG_DG3 ? sh.d3 : p.W;
  bool vec4 = (p.W % 4) == 0 && (out_inner % 4) == 0;
  long long max_count = 0, max_seg = 0;
  for (int t = 0; t < b.T; ++t) {
    const TTDev &d = b.host[t];
    const float *src = kind == SEG_GAGG ? d.grad_out : (kind == SEG_DG3 ? d.plan.t3buf : d.plan.t1buf);
    // the buffer the final stores go to: with the fused update, the core itself
    const float *out = kind == SEG_GAGG ? d.plan.gagg
                                        : (kind == SEG_DG3 ? (d.fused ? d.g[2] : d.dg[2]) : (d.fused ? d.g[0] : d.dg[0]));
    vec4 = vec4 && ((uintptr_t)src % 16) == 0 && ((uintptr_t)out % 16) == 0;
    const long long cnt = kind == SEG_GAGG ? d.nnz : (kind == SEG_DG3 ? d.plan.max_rows : d.plan.max_prefixes);
    const long long nseg = (kind == SEG_GAGG || d.fused) ? 0 : (kind == SEG_DG3 ? d.sh.n3 : d.sh.n1);
    if (cnt > max_count) max_count = cnt;
    if (nseg > max_seg) max_seg = nseg;
  }
  p.chunk = chunk > 0 ? chunk : seg_chunk_for(max_count);
  p.vec = vec4 ? 4 : 1;
  p.lanes = 1;
  while (p.lanes < TT_WAVE && p.lanes * p.vec < p.W) p.lanes <<= 1;
  p.groups = TT_BLOCK / p.lanes;
  p.nchunks = tt_ceil_div(max_count, p.chunk);
  p.blocks1 = tt_ceil_div(p.nchunks, p.groups);
  if (p.blocks1 > 8192) p.blocks1 = 8192;
  p.blocks2 = p.nchunks > max_seg ? p.nchunks : max_seg;  // dense kinds also zero-fill empty segments
  return p;
}

// One segmented sum, or (kind_b >= 0) two of the same launch shape in the same two launches.
static tt_status seg_launch(const TTBatch &b, const SegParams &pa, int kind, const SegParams *pb, int kind_b,
                            int prof_kernel, hipStream_t s) {
  TTProfScope prof(&b.host[0].plan, prof_kernel, s);  // both stages
  const size_t lds = sizeof(float) * (size_t)pa.groups * pa.W;
  SegLaunch L1 = {kind, pa.chunk, pa.blocks1, pb ? kind_b : -1, pb ? pb->chunk : 0};
  const long long g1 = pa.blocks1 + (pb ? pb->blocks1 : 0);
  if (g1 > 0) {
    if (pa.vec == 4) TT_LAUNCH_T(k_seg_stage1, 4, g1, TT_BLOCK, lds, s, b, L1, pa.lanes);
    else TT_LAUNCH_T(k_seg_stage1, 1, g1, TT_BLOCK, lds, s, b, L1, pa.lanes);
  }
  SegLaunch L2 = L1;
  L2.blocks = (int)pa.blocks2;
  const long long g2 = pa.blocks2 + (pb ? pb->blocks2 : 0);
  if (g2 > 0) {
    if (pa.vec == 4) TT_LAUNCH_T(k_seg_stage2, 4, g2, TT_BLOCK, lds, s, b, L2, pa.lanes);
    else TT_LAUNCH_T(k_seg_stage2, 1, g2, TT_BLOCK, lds, s, b, L2, pa.lanes);
  }
  return tt_launch_status();
}

tt_status seg_sum(const TTBatch &b, int kind, int chunk, int prof_kernel, hipStream_t s) {
  const SegParams p = seg_params(b, kind, chunk);
  return seg_launch(b, p, kind, nullptr, -1, prof_kernel, s);
}

#ifndef TT_SEG_WHOLE_UNROLL
#define TT_SEG_WHOLE_UNROLL TT_SEG_UNROLL  // gathers a lane group of the whole-segment kernel keeps in flight
#endif
// Whole segments: ONE launch for the core-2 and the core-0 reduction.  The first nseg_a * parts_a
// workgroups serve core 2 (rows that share i3: the index split spreads them evenly), the rest core 0,
// `parts` workgroups per segment, each summing its own range of the vector's columns.  Cutting by
// columns gives a long segment more lane groups -- more gathers in flight -- without a second stage:
// a table with few i3 values has few, long core-2 segments, and under a skewed access distribution the
// distinct prefixes pile up under the first few i1 (up to n2 prefixes times the strips each).
// The lane groups of a workgroup take the segment's positions round-robin, TT_SEG_UNROLL gathers in
// flight each, and their sums are added in group order through LDS, so the result does not depend on
// timing.  (The lookups of one hot row can be a fifth of a batch, which is why the gradient merge
// keeps the two-stage sum.)  A long segment is summed by its workgroups alone: correct, only slow.
template <bool BATCHED, int VEC>
__global__ void __launch_bounds__(TT_BLOCK)
k_seg_whole(TTArg<BATCHED> arg, int nseg_a, int lanes_a, int parts_a, int lanes_b, int parts_b) {
  const TTDev &d = arg.get();
  const bool second = (int)blockIdx.x >= nseg_a * parts_a;
  const SegView sv = seg_view(d, second ? SEG_DG1 : SEG_DG3);
  const int parts = second ? parts_b : parts_a;
  const int wg = second ? (int)blockIdx.x - nseg_a * parts_a : (int)blockIdx.x;
  const int s = wg / parts, part = wg - s * parts;
  if (s >= sv.nseg) return;  // uniform: a table of the batch with fewer segments
  const int lanes = second ? lanes_b : lanes_a;
  const int W = sv.W, nsub = sv.nsub, out_inner = sv.out_inner, nseg = sv.nseg;
  const int Wp = W / parts, e0 = part * Wp;  // this workgroup's columns
  const int32_t *__restrict__ gidx = sv.gidx, *__restrict__ seg_off = sv.seg_off;
  const float *__restrict__ src = sv.src;
  float *__restrict__ out = sv.out;
  const int groups = blockDim.x / lanes, g = threadIdx.x / lanes, lane = threadIdx.x - g * lanes;
  extern __shared__ float red[];  // [groups][Wp]
  const int a = seg_off[s], b = seg_off[s + 1];
  if (a == b) {  // uniform: an empty segment (a slice no lookup touched)
    if (sv.dense && g == 0) {
      Vec<VEC> z;
      z.zero();
      for (int e = lane * VEC; e < Wp; e += lanes * VEC) z.store(out + seg_out_index(s, e0 + e, out_inner, nseg));
    }
    return;
  }
  auto load_pos = [&](int pos, int e, Vec<VEC> &x) {
    const int row = gidx ? gidx[pos] : pos;
    x.load_stream(src + (size_t)row * nsub * W + e0 + e);  // hand-off buffers: every vector is read once
    for (int t = 1; t < nsub; ++t) {
      Vec<VEC> y;
      y.load_stream(src + ((size_t)row * nsub + t) * W + e0 + e);
      x.add(y);
    }
  };
  for (int e = lane * VEC; e < Wp; e += lanes * VEC) {
    Vec<VEC> acc;
    acc.zero();
    int pos = a + g;
    for (; pos + (TT_SEG_WHOLE_UNROLL - 1) * groups < b; pos += TT_SEG_WHOLE_UNROLL * groups) {
      Vec<VEC> x[TT_SEG_WHOLE_UNROLL];
#pragma unroll
      for (int k = 0; k < TT_SEG_WHOLE_UNROLL; ++k) load_pos(pos + k * groups, e, x[k]);
#pragma unroll
      for (int k = 0; k < TT_SEG_WHOLE_UNROLL; ++k) acc.add(x[k]);
    }
    for (; pos < b; pos += groups) {
      Vec<VEC> x;
      load_pos(pos, e, x);
      acc.add(x);
    }
    acc.store(red + (size_t)g * Wp + e);
  }
  __syncthreads();
  if (g == 0)
    for (int e = lane * VEC; e < Wp; e += lanes * VEC) {
      Vec<VEC> acc, x;
      acc.load(red + e);
      for (int k = 1; k < groups; ++k) {
        x.load(red + (size_t)k * Wp + e);
        acc.add(x);
      }
      float *dst = out + seg_out_index(s, e0 + e, out_inner, nseg);
      if (sv.fused) acc.store_sgd(dst, sv.lr); else acc.store(dst);
    }
}

#ifndef TT_SEG_WHOLE_PARTS
#define TT_SEG_WHOLE_PARTS 8  // column parts of a core-0 segment
#endif
#ifndef TT_SEG_WHOLE_MAX_AVG
#define TT_SEG_WHOLE_MAX_AVG 4096  // positions per segment (capacity / segments) up to which whole segments are used
#endif

// The core-2 and core-0 reductions are independent.  With segments of moderate length they take one
// launch of whole-segment workgroups; otherwise the two-stage sum, sharing its launches when their
// vectors have the same width (the smaller one would otherwise pay two launches for a few workgroups).
tt_status seg_sum_dg3_dg1(const TTBatch &b, hipStream_t s) {
  const SegParams p3 = seg_params(b, SEG_DG3, 0), p1 = seg_params(b, SEG_DG1, 0);
  bool whole = p3.vec == p1.vec;
  for (int t = 0; t < b.T && whole; ++t) {
    const TTDev &d = b.host[t];
    whole = d.plan.max_rows / d.sh.n3 <= TT_SEG_WHOLE_MAX_AVG &&
            d.plan.max_prefixes * d.strips / d.sh.n1 <= TT_SEG_WHOLE_MAX_AVG;
  }
  if (whole) {
    const long long n3max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n3; });
    const long long n1max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n1; });
    // column parts per segment: core 0 as many (at most TT_SEG_WHOLE_PARTS) as leave a part 8 lanes wide;
    // core 2 only as many as bring its workgroups to about two per compute unit
    auto parts_for = [](const SegParams &p, int want) {
      int parts = 1;
      while (parts * 2 <= want && p.W % (parts * 2 * p.vec) == 0 && p.W / (parts * 2 * p.vec) >= 8) parts *= 2;
      return parts;
    };
    auto lanes_for = [](const SegParams &p, int parts) {
      int lanes = 1;
      while (lanes < TT_WAVE && lanes * p.vec < p.W / parts) lanes <<= 1;
      return lanes;
    };
    const int parts3 = parts_for(p3, tt_ceil_div(512, n3max) < TT_SEG_WHOLE_PARTS ? tt_ceil_div(512, n3max) : TT_SEG_WHOLE_PARTS);
    const int parts1 = parts_for(p1, TT_SEG_WHOLE_PARTS);
    const int lanes3 = lanes_for(p3, parts3), lanes1 = lanes_for(p1, parts1);
    const size_t g3 = (size_t)(TT_BLOCK / lanes3) * (p3.W / parts3), g1 = (size_t)(TT_BLOCK / lanes1) * (p1.W / parts1);
    const size_t lds = sizeof(float) * (g3 > g1 ? g3 : g1);
    const long long grid = n3max * parts3 + n1max * parts1;
    if (p3.vec == 4) TT_LAUNCH_T(k_seg_whole, 4, grid, TT_BLOCK, lds, s, b, (int)n3max, lanes3, parts3, lanes1, parts1);
    else TT_LAUNCH_T(k_seg_whole, 1, grid, TT_BLOCK, lds, s, b, (int)n3max, lanes3, parts3, lanes1, parts1);
    return tt_launch_status();
  }
  if (p3.W == p1.W && p3.vec == p1.vec && p3.lanes == p1.lanes && p3.blocks1 > 0 && p1.blocks1 > 0)
    return seg_launch(b, p3, SEG_DG3, &p1, SEG_DG1, -1, s);
  tt_status st = seg_launch(b, p3, SEG_DG3, nullptr, -1, -1, s);
  if (st != TT_OK) return st;
  return seg_launch(b, p1, SEG_DG1, nullptr, -1, -1, s);
}

// ------------------------------------------------------------------ per-prefix contractions
// Workgroup per distinct prefix q.
// LDS (floats): g1s[S1] | p12[d1*d2*R2p] | hs[P] | gs[D] | g3s[S3]
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_prefix(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int32_t *__restrict__ counts = d.plan.counts, *__restrict__ uniq_pref = d.plan.uniq_pref,
                *__restrict__ pref_seg = d.plan.pref_seg, *__restrict__ uniq_row = d.plan.uniq_row;
  const float *__restrict__ gagg = d.plan.gagg;
  float *__restrict__ t3buf = d.plan.t3buf, *__restrict__ hbuf = d.plan.hbuf,
        *__restrict__ t1buf = d.plan.t1buf;
  extern __shared__ float lds[];
  float *g1s = lds, *p12 = g1s + sh.S1, *hs = p12 + sh.d1 * sh.d2 * sh.R2p, *gs = hs + sh.P,
        *g3s = gs + sh.D;
  const int up = counts[1];
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;
  for (int q = blockIdx.x; q < up; q += gridDim.x) {
    const int p = uniq_pref[q], i1 = p / sh.n2, i2 = p - i1 * sh.n2;
    for (int e = threadIdx.x; e < sh.S1; e += blockDim.x) g1s[e] = g1[(size_t)i1 * sh.S1 + e];
    for (int o = threadIdx.x; o < sh.P; o += blockDim.x) hs[o] = 0.f;
    __syncthreads();
    // P12[j1][j2][r2] = sum_r1 G1[i1][j1][r1] G2[r1][i2][j2][r2]
    for (int o = threadIdx.x; o < sh.P; o += blockDim.x) {
      const int j1 = o / sh.S2, c = o - j1 * sh.S2;
      const float *col = g2 + (size_t)i2 * sh.S2 + c;
      float acc = 0.f;
      for (int r1 = 0; r1 < sh.R1; ++r1)
        acc = fmaf(g1s[j1 * sh.R1 + r1], col[(size_t)r1 * sh.n2 * sh.S2], acc);
      p12[(j1 * sh.d2 + c / sh.R2) * sh.R2p + c % sh.R2] = acc;
    }
    const int u0 = pref_seg[q], u1 = pref_seg[q + 1];
    for (int u = u0; u < u1; ++u) {
      const int i3 = uniq_row[u] % sh.n3;
      __syncthreads();  // previous row's readers are done; p12 / hs initialisation is visible
      for (int e = threadIdx.x; e < sh.D; e += blockDim.x) gs[e] = gagg[(size_t)u * sh.D + e];
      for (int e = threadIdx.x; e < sh.S3; e += blockDim.x) {
        const int r2 = e / sh.d3, j3 = e - r2 * sh.d3;
        g3s[e] = g3[((size_t)r2 * sh.n3 + i3) * sh.d3 + j3];
      }
      __syncthreads();
      // core-2 contribution of this row: T3[r2][j3] = sum_{j1,j2} P12[j1][j2][r2] g[j1][j2][j3]
      for (int o = threadIdx.x; o < sh.S3; o += blockDim.x) {
        const int r2 = o / sh.d3, j3 = o - r2 * sh.d3;
        float acc = 0.f;
        for (int jj = 0; jj < sh.d1 * sh.d2; ++jj)
          acc = fmaf(p12[jj * sh.R2p + r2], gs[jj * sh.d3 + j3], acc);
        t3buf[(size_t)u * sh.S3 + o] = acc;
      }
      // right partial: H[j1][j2][r2] += sum_j3 g[j1][j2][j3] G3[r2][i3][j3]
      for (int o = threadIdx.x; o < sh.P; o += blockDim.x) {
        const int jj = o / sh.R2, r2 = o - jj * sh.R2;
        float acc = 0.f;
        for (int j3 = 0; j3 < sh.d3; ++j3) acc = fmaf(gs[jj * sh.d3 + j3], g3s[r2 * sh.d3 + j3], acc);
        hs[o] += acc;
      }
    }
    __syncthreads();
    for (int o = threadIdx.x; o < sh.P; o += blockDim.x) hbuf[(size_t)q * sh.P + o] = hs[o];
    // core-0 contribution: T1[j1][r1] = sum_{j2,r2} H[j1][j2][r2] G2[r1][i2][j2][r2]
    // one wavefront per r1: coalesced read of the G2 row, shuffle reduction over (j2,r2)
    for (int r1 = wave; r1 < sh.R1; r1 += blockDim.x / TT_WAVE) {
      const float *rowp = g2 + ((size_t)r1 * sh.n2 + i2) * sh.S2;
      for (int j1 = 0; j1 < sh.d1; ++j1) {
        float part = 0.f;
        for (int c = lane; c < sh.S2; c += TT_WAVE) part = fmaf(hs[j1 * sh.S2 + c], rowp[c], part);
        part = tt_wave_sum(part);
        if (lane == 0) t1buf[(size_t)q * sh.S1 + j1 * sh.R1 + r1] = part;
      }
    }
    __syncthreads();
  }
}

// Core-1 gradient: dG2[r1][i2][j2][r2] = sum over the prefixes (i1,i2) of the batch of
// sum_j1 G1[i1][j1][r1] H[(i1,i2)][j1][j2][r2].  Workgroup (i2, column tile, r1 tile); thread
// owns one (j2,r2) column and RT values of r1; prefixes are visited in increasing i1.
#define TT_DG2_RT 8
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_dg2(TTArg<BATCHED> a, int col_tiles) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ hbuf = d.plan.hbuf;
  const int32_t *__restrict__ uniq_pref = d.plan.uniq_pref, *__restrict__ prefs_by_i2 = d.plan.prefs_by_i2,
                *__restrict__ i2_seg = d.plan.i2_seg;
  float *__restrict__ dg2 = d.fused ? const_cast<float *>(d.g[1]) : d.dg[1];
  const int fused = d.fused;
  const float lr = d.lr;
  // grid.x enumerates (i2, column tile, r1 tile); grid.y is the table in a batched launch
  const int r1_tiles = (sh.R1 + TT_DG2_RT - 1) / TT_DG2_RT;
  if ((int)blockIdx.x >= sh.n2 * col_tiles * r1_tiles) return;
  const int bz = blockIdx.x % r1_tiles, by = (blockIdx.x / r1_tiles) % col_tiles,
            bx = blockIdx.x / (r1_tiles * col_tiles);
  const int i2 = bx, c = by * TT_BLOCK + threadIdx.x, r1b = bz * TT_DG2_RT;
  if (c >= sh.S2) return;
  float acc[TT_DG2_RT];
#pragma unroll
  for (int k = 0; k < TT_DG2_RT; ++k) acc[k] = 0.f;
  const int s0 = i2_seg[i2], s1 = i2_seg[i2 + 1];
  if (fused && s0 == s1) return;  // untouched slice: nothing to apply
  for (int s = s0; s < s1; ++s) {
    const int q = prefs_by_i2[s], i1 = uniq_pref[q] / sh.n2;
    for (int j1 = 0; j1 < sh.d1; ++j1) {
      const float h = hbuf[(size_t)q * sh.P + j1 * sh.S2 + c];
      const float *gp = g1 + (size_t)i1 * sh.S1 + j1 * sh.R1 + r1b;
#pragma unroll
      for (int k = 0; k < TT_DG2_RT; ++k)
        if (r1b + k < sh.R1) acc[k] = fmaf(gp[k], h, acc[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < TT_DG2_RT; ++k)
    if (r1b + k < sh.R1) {
      float *dst = dg2 + ((size_t)(r1b + k) * sh.n2 + i2) * sh.S2 + c;
      *dst = fused ? fmaf(-lr, acc[k], *dst) : acc[k];
    }
}

// ------------------------------------------------------------------ naive arm
template <bool BATCHED>
__global__ void k_fill_zero_core(TTArg<BATCHED> a, int k) {
  const TTDev &d = a.get();
  float *__restrict__ p = d.dg[k];
  const size_t count = k == 0 ? (size_t)d.sh.n1 * d.sh.S1
                              : (k == 1 ? (size_t)d.sh.R1 * d.sh.n2 * d.sh.S2 : (size_t)d.sh.n3 * d.sh.S3);
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
       e += (size_t)gridDim.x * blockDim.x)
    p[e] = 0.f;
}

// Workgroup per lookup, no dedup, floating-point atomics into the core gradients.
// LDS: g1s[S1] | p12[d1*d2*R2p] | hs[P] | gs[D] | g3s[S3]
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_naive(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int64_t *__restrict__ indices = d.indices, *__restrict__ offsets = d.offsets;
  const int nnz = d.nnz, num_bags = d.num_bags;
  const float *__restrict__ grad_out = d.grad_out;
  float *__restrict__ dg1 = d.dg[0], *__restrict__ dg2 = d.dg[1], *__restrict__ dg3 = d.dg[2];
  extern __shared__ float lds[];
  float *g1s = lds, *p12 = g1s + sh.S1, *hs = p12 + sh.d1 * sh.d2 * sh.R2p, *gs = hs + sh.P,
        *g3s = gs + sh.D;
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;
  for (int l = blockIdx.x; l < nnz; l += gridDim.x) {
    const long long row = indices[l];
    if (row < 0 || row >= sh.num_rows) continue;  // uniform
    int lo = 0, hi = num_bags;  // bag holding position l
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (offsets[mid] <= (long long)l) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int i3 = (int)(row % sh.n3), p = (int)(row / sh.n3), i1 = p / sh.n2, i2 = p - i1 * sh.n2;
    __syncthreads();
    for (int e = threadIdx.x; e < sh.S1; e += blockDim.x) g1s[e] = g1[(size_t)i1 * sh.S1 + e];
    for (int e = threadIdx.x; e < sh.D; e += blockDim.x) gs[e] = grad_out[(size_t)b * sh.D + e];
    for (int e = threadIdx.x; e < sh.S3; e += blockDim.x) {
      const int r2 = e / sh.d3, j3 = e - r2 * sh.d3;
      g3s[e] = g3[((size_t)r2 * sh.n3 + i3) * sh.d3 + j3];
    }
    __syncthreads();
    for (int o = threadIdx.x; o < sh.P; o += blockDim.x) {
      const int j1 = o / sh.S2, c = o - j1 * sh.S2;
      const float *col = g2 + (size_t)i2 * sh.S2 + c;
      float acc = 0.f;
      for (int r1 = 0; r1 < sh.R1; ++r1)
        acc = fmaf(g1s[j1 * sh.R1 + r1], col[(size_t)r1 * sh.n2 * sh.S2], acc);
      p12[(j1 * sh.d2 + c / sh.R2) * sh.R2p + c % sh.R2] = acc;
      // right partial u[j1][j2][r2] = sum_j3 g[j1][j2][j3] G3[r2][i3][j3]  (o indexes [jj][r2])
      const int jj = o / sh.R2, r2 = o - jj * sh.R2;
      float h = 0.f;
      for (int j3 = 0; j3 < sh.d3; ++j3) h = fmaf(gs[jj * sh.d3 + j3], g3s[r2 * sh.d3 + j3], h);
      hs[o] = h;
    }
    __syncthreads();
    for (int o = threadIdx.x; o < sh.S3; o += blockDim.x) {
      const int r2 = o / sh.d3, j3 = o - r2 * sh.d3;
      float acc = 0.f;
      for (int jj = 0; jj < sh.d1 * sh.d2; ++jj)
        acc = fmaf(p12[jj * sh.R2p + r2], gs[jj * sh.d3 + j3], acc);
      atomicAdd(dg3 + ((size_t)r2 * sh.n3 + i3) * sh.d3 + j3, acc);
    }
    for (int o = threadIdx.x; o < sh.R1 * sh.S2; o += blockDim.x) {
      const int r1 = o / sh.S2, c = o - r1 * sh.S2;
      float acc = 0.f;
      for (int j1 = 0; j1 < sh.d1; ++j1) acc = fmaf(g1s[j1 * sh.R1 + r1], hs[j1 * sh.S2 + c], acc);
      atomicAdd(dg2 + ((size_t)r1 * sh.n2 + i2) * sh.S2 + c, acc);
    }
    for (int r1 = wave; r1 < sh.R1; r1 += blockDim.x / TT_WAVE) {
      const float *rowp = g2 + ((size_t)r1 * sh.n2 + i2) * sh.S2;
      for (int j1 = 0; j1 < sh.d1; ++j1) {
        float part = 0.f;
        for (int c = lane; c < sh.S2; c += TT_WAVE) part = fmaf(hs[j1 * sh.S2 + c], rowp[c], part);
        part = tt_wave_sum(part);
        if (lane == 0) atomicAdd(dg1 + (size_t)i1 * sh.S1 + j1 * sh.R1 + r1, part);
      }
    }
  }
}

// ------------------------------------------------------------------ gradient-descent update
template <bool BATCHED>
__global__ void k_sgd_dense(TTArg<BATCHED> a, int k) {
  const TTDev &d = a.get();
  float *__restrict__ g = const_cast<float *>(d.g[k]);
  const float *__restrict__ dg = d.dg[k];
  const float lr = d.lr;
  const size_t count = k == 0 ? (size_t)d.sh.n1 * d.sh.S1
                              : (k == 1 ? (size_t)d.sh.R1 * d.sh.n2 * d.sh.S2 : (size_t)d.sh.n3 * d.sh.S3);
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
       e += (size_t)gridDim.x * blockDim.x)
    g[e] = fmaf(-lr, dg[e], g[e]);
}

// Workgroup per slice of any of the three cores; untouched slices (empty range) are skipped.
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_sgd_touched(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  float *__restrict__ g1 = const_cast<float *>(d.g[0]), *__restrict__ g2 = const_cast<float *>(d.g[1]),
        *__restrict__ g3 = const_cast<float *>(d.g[2]);
  const float *__restrict__ dg1 = d.dg[0], *__restrict__ dg2 = d.dg[1], *__restrict__ dg3 = d.dg[2];
  const int32_t *__restrict__ i1_seg = d.plan.i1_seg, *__restrict__ i2_seg = d.plan.i2_seg,
                *__restrict__ i3_seg = d.plan.i3_seg;
  const float lr = d.lr;
  int s = blockIdx.x;
  if (s >= sh.n1 + sh.n2 + sh.n3) return;  // a narrower table of the batch
  if (s < sh.n1) {
    if (i1_seg[s] == i1_seg[s + 1]) return;
    for (int e = threadIdx.x; e < sh.S1; e += blockDim.x) {
      const size_t a = (size_t)s * sh.S1 + e;
      g1[a] = fmaf(-lr, dg1[a], g1[a]);
    }
    return;
  }
  s -= sh.n1;
  if (s < sh.n2) {
    if (i2_seg[s] == i2_seg[s + 1]) return;
    for (int e = threadIdx.x; e < sh.R1 * sh.S2; e += blockDim.x) {
      const int r1 = e / sh.S2, c = e - r1 * sh.S2;
      const size_t a = ((size_t)r1 * sh.n2 + s) * sh.S2 + c;
      g2[a] = fmaf(-lr, dg2[a], g2[a]);
    }
    return;
  }
  s -= sh.n2;
  if (i3_seg[s] == i3_seg[s + 1]) return;
  for (int e = threadIdx.x; e < sh.S3; e += blockDim.x) {
    const int r2 = e / sh.d3, j3 = e - r2 * sh.d3;
    const size_t a = ((size_t)r2 * sh.n3 + s) * sh.d3 + j3;
    g3[a] = fmaf(-lr, dg3[a], g3[a]);
  }
}

size_t bwd_lds_bytes(const TTShape &sh) {
  return sizeof(float) * ((size_t)sh.S1 + (size_t)sh.d1 * sh.d2 * sh.R2p + sh.P + sh.D + sh.S3);
}

long long core_len(const TTShape &sh, int k) {
  if (k == 0) return (long long)sh.n1 * sh.S1;
  if (k == 1) return (long long)sh.R1 * sh.n2 * sh.S2;
  return (long long)sh.n3 * sh.S3;
}

}  // namespace

tt_status ttk_backward_plan(const TTBatch &b, hipStream_t s) {
  const TTShape &sh = b.host[0].sh;
  tt_status st;
  // 1. merge output gradients per distinct row
  if ((st = seg_sum(b, SEG_GAGG, 0, TT_KERNEL_GRAD_MERGE, s)) != TT_OK) return st;
  // 2. per-prefix contractions
  const bool mfma = ttk_batch_mfma(b);
  const long long max_pref = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_prefixes; });
  if (mfma) {
    if ((st = ttk_backward_mfma(b, s)) != TT_OK) return st;
  } else if (max_pref > 0) {
    const long long blocks = max_pref < 4096 ? max_pref : 4096;
    TTProfScope prof(&b.host[0].plan, TT_KERNEL_BWD_CONTRACT, s);
    TT_LAUNCH(k_bwd_prefix, blocks, TT_BLOCK, bwd_lds_bytes(sh), s, b);
  }
  // 3. core 1: per-i2 accumulation over prefixes (inside the matrix-core kernel, else here).  It
  //    reads core 0, so with the fused update it has to run before the core-0 reduction below.
  if (!mfma) {
    const int col_tiles = tt_ceil_div(sh.S2, TT_BLOCK), r1_tiles = tt_ceil_div(sh.R1, TT_DG2_RT);
    const long long n2max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n2; });
    TT_LAUNCH(k_bwd_dg2, n2max * col_tiles * r1_tiles, TT_BLOCK, 0, s, b, col_tiles);
  }
  // 4. core 2: sum the per-row contributions of all rows sharing i3; core 0: sum the per-prefix
  //    contributions of all prefixes sharing i1 (contiguous)
  if ((st = seg_sum_dg3_dg1(b, s)) != TT_OK) return st;
  return tt_launch_status();
}

tt_status ttk_backward_naive(const TTBatch &b, hipStream_t s) {
  for (int k = 0; k < 3; ++k) {
    const long long len = tt_batch_max(b, [k](const TTDev &d) { return core_len(d.sh, k); });
    int blocks = tt_ceil_div(len, TT_BLOCK * 4);
    if (blocks > 4096) blocks = 4096;
    TT_LAUNCH(k_fill_zero_core, blocks, TT_BLOCK, 0, s, b, k);
  }
  const long long max_nnz = tt_batch_max(b, [](const TTDev &d) { return (long long)d.nnz; });
  if (max_nnz > 0) {
    const long long blocks = max_nnz < 65536 ? max_nnz : 65536;
    TT_LAUNCH(k_bwd_naive, blocks, TT_BLOCK, bwd_lds_bytes(b.host[0].sh), s, b);
  }
  return tt_launch_status();
}

tt_status ttk_sgd(const TTBatch &b, bool touched_only, hipStream_t s) {
  if (touched_only) {
    const long long slices = tt_batch_max(b, [](const TTDev &d) {
      return (long long)d.sh.n1 + d.sh.n2 + d.sh.n3; });
    TTProfScope prof(&b.host[0].plan, TT_KERNEL_SGD, s);
    TT_LAUNCH(k_sgd_touched, slices, TT_BLOCK, 0, s, b);
  } else {
    for (int k = 0; k < 3; ++k) {
      const long long len = tt_batch_max(b, [k](const TTDev &d) { return core_len(d.sh, k); });
      int blocks = tt_ceil_div(len, TT_BLOCK * 4);
      if (blocks > 4096) blocks = 4096;
      TT_LAUNCH(k_sgd_dense, blocks, TT_BLOCK, 0, s, b, k);
    }
  }
  return tt_launch_status();
}
