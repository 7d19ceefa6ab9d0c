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
  __device__ __forceinline__ void store(float *p) const {
    if (VEC == 4) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1 % VEC], v[2 % VEC], v[3 % VEC]);
    else *p = v[0];
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

template <int VEC>
__global__ void __launch_bounds__(TT_BLOCK)
k_seg_stage1(int W, int lanes, const int32_t *__restrict__ count_ptr,
             const int32_t *__restrict__ seg_src, int seg_div, const int32_t *__restrict__ gidx,
             const int32_t *__restrict__ seg_off, const float *__restrict__ src, int nsub,
             float *__restrict__ out, int out_inner, int nseg, float *__restrict__ partial,
             int chunk) {
  const int M = *count_ptr;
  const int nchunks = (M + chunk - 1) / chunk;
  const int groups = blockDim.x / lanes, g = threadIdx.x / lanes, lane = threadIdx.x - g * lanes;
  for (int c = blockIdx.x * groups + g; c < nchunks; c += gridDim.x * groups) {
    const int lo = c * chunk, hi = lo + chunk, end = hi < M ? hi : M;
    for (int e = lane * VEC; e < W; e += lanes * VEC) {
      Vec<VEC> acc;
      acc.zero();
      int cur = -1;
      auto flush = [&]() {
        const int a = seg_off[cur], b = seg_off[cur + 1];
        if (a >= lo && b <= hi) acc.store(out + seg_out_index(cur, e, out_inner, nseg));
        else acc.store(partial + ((size_t)c * 2 + (a < lo ? 0 : 1)) * W + e);
      };
      int pos = lo;
      for (; pos + TT_SEG_UNROLL <= end; pos += TT_SEG_UNROLL) {  // independent gathers in flight,
        int sg[TT_SEG_UNROLL];                                    // added in position order
        Vec<VEC> x[TT_SEG_UNROLL];
#pragma unroll
        for (int k = 0; k < TT_SEG_UNROLL; ++k) {
          sg[k] = seg_src[pos + k] / seg_div;
          const int row = gidx ? gidx[pos + k] : pos + k;
          x[k].load(src + (size_t)row * nsub * W + e);
          for (int t = 1; t < nsub; ++t) {
            Vec<VEC> y;
            y.load(src + ((size_t)row * nsub + t) * W + e);
            x[k].add(y);
          }
        }
#pragma unroll
        for (int k = 0; k < TT_SEG_UNROLL; ++k) {
          if (sg[k] != cur) {
            if (cur >= 0) flush();
            cur = sg[k];
            acc.zero();
          }
          acc.add(x[k]);
        }
      }
      for (; pos < end; ++pos) {
        const int sgk = seg_src[pos] / seg_div;
        const int row = gidx ? gidx[pos] : pos;
        Vec<VEC> x;
        x.load(src + (size_t)row * nsub * W + e);
        for (int t = 1; t < nsub; ++t) {
          Vec<VEC> y;
          y.load(src + ((size_t)row * nsub + t) * W + e);
          x.add(y);
        }
        if (sgk != cur) {
          if (cur >= 0) flush();
          cur = sgk;
          acc.zero();
        }
        acc.add(x);
      }
      if (cur >= 0) flush();
    }
  }
}

// Stage 2: workgroup per chunk.  The chunk in which a multi-chunk segment begins owns it and adds
// its own slot-1 partial and the slot-0 partials of the following chunks, in chunk order.
// With `dense`, workgroup c also zero-fills segment c if it is empty.
// LDS: red[groups][W]
template <int VEC>
__global__ void __launch_bounds__(TT_BLOCK)
k_seg_stage2(int W, int lanes, const int32_t *__restrict__ count_ptr,
             const int32_t *__restrict__ seg_src, int seg_div,
             const int32_t *__restrict__ seg_off, float *__restrict__ out, int out_inner,
             int nseg, const float *__restrict__ partial, int dense, int chunk) {
  extern __shared__ float red[];
  const int M = *count_ptr;
  const int nchunks = (M + chunk - 1) / chunk;
  const int c = blockIdx.x;
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
  for (int e = lane * VEC; e < W; e += lanes * VEC) {
    Vec<VEC> acc;
    acc.zero();
    if (g < groups) {
      int cc = c + 1 + g;
      for (; cc + 3 * groups <= c1; cc += 4 * groups) {
        Vec<VEC> x[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k].load(partial + ((size_t)(cc + k * groups) * 2) * W + e);
#pragma unroll
        for (int k = 0; k < 4; ++k) acc.add(x[k]);
      }
      for (; cc <= c1; cc += groups) {
        Vec<VEC> x;
        x.load(partial + ((size_t)cc * 2) * W + e);
        acc.add(x);
      }
      acc.store(red + (size_t)g * W + e);
    }
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
      acc.store(out + seg_out_index(s, e, out_inner, nseg));
    }
  }
}

struct SegArgs {
  int W;
  const int32_t *count_ptr;  // device: number of positions
  int64_t max_count;         // host upper bound of *count_ptr
  const int32_t *seg_src;
  int seg_div;
  const int32_t *gidx;
  const int32_t *seg_off;
  const float *src;
  int nsub;  // vectors per position
  float *out;
  int out_inner;
  int nseg;   // number of segments for the output layout / dense zero fill
  int dense;
  float *partial;
  int chunk;            // positions per stage-1 chunk (>= TT_SEG_MIN_CHUNK)
  const tt_plan *plan;  // for the optional timing scope
  int prof_kernel;      // kernel id of stage 1, or -1
};

tt_status seg_sum(const SegArgs &a, hipStream_t s) {
  const bool vec4 = (a.W % 4) == 0 && (a.out_inner % 4) == 0 && ((uintptr_t)a.src % 16) == 0 &&
                    ((uintptr_t)a.out % 16) == 0;
  const int vec = vec4 ? 4 : 1;
  int lanes = 1;
  while (lanes < TT_WAVE && lanes * vec < a.W) lanes <<= 1;
  const int groups = TT_BLOCK / lanes;
  const int nchunks = tt_ceil_div(a.max_count, a.chunk);
  if (nchunks > 0) {
    int blocks = tt_ceil_div(nchunks, groups);
    if (blocks > 8192) blocks = 8192;
    TTProfScope prof(a.plan, a.prof_kernel, s);
    if (vec4)
      hipLaunchKernelGGL(k_seg_stage1<4>, dim3(blocks), dim3(TT_BLOCK), 0, s, a.W, lanes,
                         a.count_ptr, a.seg_src, a.seg_div, a.gidx, a.seg_off, a.src, a.nsub, a.out,
                         a.out_inner, a.nseg, a.partial, a.chunk);
    else
      hipLaunchKernelGGL(k_seg_stage1<1>, dim3(blocks), dim3(TT_BLOCK), 0, s, a.W, lanes,
                         a.count_ptr, a.seg_src, a.seg_div, a.gidx, a.seg_off, a.src, a.nsub, a.out,
                         a.out_inner, a.nseg, a.partial, a.chunk);
  }
  int blocks2 = nchunks;
  if (a.dense && a.nseg > blocks2) blocks2 = a.nseg;
  if (blocks2 > 0) {
    const size_t lds = sizeof(float) * (size_t)groups * a.W;
    if (vec4)
      hipLaunchKernelGGL(k_seg_stage2<4>, dim3(blocks2), dim3(TT_BLOCK), lds, s, a.W, lanes,
                         a.count_ptr, a.seg_src, a.seg_div, a.seg_off, a.out, a.out_inner, a.nseg,
                         a.partial, a.dense, a.chunk);
    else
      hipLaunchKernelGGL(k_seg_stage2<1>, dim3(blocks2), dim3(TT_BLOCK), lds, s, a.W, lanes,
                         a.count_ptr, a.seg_src, a.seg_div, a.seg_off, a.out, a.out_inner, a.nseg,
                         a.partial, a.dense, a.chunk);
  }
  return tt_launch_status();
}

// ------------------------------------------------------------------ per-prefix contractions
// Workgroup per distinct prefix q.
// LDS (floats): g1s[S1] | p12[d1*d2*R2p] | hs[P] | gs[D] | g3s[S3]
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_prefix(TTShape sh, const float *__restrict__ g1, const float *__restrict__ g2,
             const float *__restrict__ g3, const int32_t *__restrict__ counts,
             const int32_t *__restrict__ uniq_pref, const int32_t *__restrict__ pref_seg,
             const int32_t *__restrict__ uniq_row, const float *__restrict__ gagg,
             float *__restrict__ t3buf, float *__restrict__ hbuf, float *__restrict__ t1buf) {
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
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_dg2(TTShape sh, const float *__restrict__ g1, const int32_t *__restrict__ uniq_pref,
          const int32_t *__restrict__ prefs_by_i2, const int32_t *__restrict__ i2_seg,
          const float *__restrict__ hbuf, float *__restrict__ dg2) {
  const int i2 = blockIdx.x, c = blockIdx.y * TT_BLOCK + threadIdx.x, r1b = blockIdx.z * TT_DG2_RT;
  if (c >= sh.S2) return;
  float acc[TT_DG2_RT];
#pragma unroll
  for (int k = 0; k < TT_DG2_RT; ++k) acc[k] = 0.f;
  const int s0 = i2_seg[i2], s1 = i2_seg[i2 + 1];
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
    if (r1b + k < sh.R1) dg2[((size_t)(r1b + k) * sh.n2 + i2) * sh.S2 + c] = acc[k];
}

// ------------------------------------------------------------------ naive arm
__global__ void k_fill_zero(float *__restrict__ p, size_t count) {
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
       e += (size_t)gridDim.x * blockDim.x)
    p[e] = 0.f;
}

// Workgroup per lookup, no dedup, floating-point atomics into the core gradients.
// LDS: g1s[S1] | p12[d1*d2*R2p] | hs[P] | gs[D] | g3s[S3]
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_naive(TTShape sh, const float *__restrict__ g1, const float *__restrict__ g2,
            const float *__restrict__ g3, const int64_t *__restrict__ indices,
            const int64_t *__restrict__ offsets, int nnz, int num_bags,
            const float *__restrict__ grad_out, float *__restrict__ dg1, float *__restrict__ dg2,
            float *__restrict__ dg3) {
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
__global__ void k_sgd_dense(float *__restrict__ g, const float *__restrict__ dg, size_t count,
                            float lr) {
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
       e += (size_t)gridDim.x * blockDim.x)
    g[e] = fmaf(-lr, dg[e], g[e]);
}

// Workgroup per slice of any of the three cores; untouched slices (empty range) are skipped.
__global__ void __launch_bounds__(TT_BLOCK)
k_sgd_touched(TTShape sh, float *__restrict__ g1, float *__restrict__ g2, float *__restrict__ g3,
              const float *__restrict__ dg1, const float *__restrict__ dg2,
              const float *__restrict__ dg3, const int32_t *__restrict__ i1_seg,
              const int32_t *__restrict__ i2_seg, const int32_t *__restrict__ i3_seg, float lr) {
  int s = blockIdx.x;
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

size_t core_len(const TTShape &sh, int k) {
  if (k == 0) return (size_t)sh.n1 * sh.S1;
  if (k == 1) return (size_t)sh.R1 * sh.n2 * sh.S2;
  return (size_t)sh.n3 * sh.S3;
}

}  // namespace

tt_status ttk_backward_plan(const TTShape &sh, const tt_table *t, const tt_plan *plan,
                            const float *grad_out, float *const dcore[3], hipStream_t s) {
  tt_status st;
  // 1. merge output gradients per distinct row
  SegArgs a1 = {sh.D, plan->counts + 2, plan->nnz, plan->slot_of_sorted, 1, plan->bag_of_sorted,
                plan->row_seg, grad_out, 1, plan->gagg, sh.D, (int)plan->max_rows, 0,
                plan->partial, 32, plan, TT_KERNEL_GRAD_MERGE};
  if ((st = seg_sum(a1, s)) != TT_OK) return st;
  // 2. per-prefix contractions
  const bool mfma = tt_mfma_enabled() && ttk_forward_mfma_supported(sh);
  const int strips = mfma ? ttk_mfma_strips(sh) : 1;
  if (mfma) {
    if ((st = ttk_backward_mfma(sh, t, plan, dcore[1], s)) != TT_OK) return st;
  } else if (plan->max_prefixes > 0) {
    long long blocks = plan->max_prefixes < 4096 ? plan->max_prefixes : 4096;
    TTProfScope prof(plan, TT_KERNEL_BWD_CONTRACT, s);
    hipLaunchKernelGGL(k_bwd_prefix, dim3((unsigned)blocks), dim3(TT_BLOCK), bwd_lds_bytes(sh), s,
                       sh, t->core[0], t->core[1], t->core[2], plan->counts, plan->uniq_pref,
                       plan->pref_seg, plan->uniq_row, plan->gagg, plan->t3buf, plan->hbuf,
                       plan->t1buf);
  }
  // 3a. core 2: sum the per-row contributions of all rows sharing i3
  SegArgs a3 = {sh.S3, plan->counts + 0, plan->max_rows, plan->i3_of_sorted, 1, plan->rows_by_i3,
                plan->i3_seg, plan->t3buf, strips, dcore[2], sh.d3, sh.n3, 1, plan->partial, TT_SEG_MIN_CHUNK, plan, -1};
  if ((st = seg_sum(a3, s)) != TT_OK) return st;
  // 3b. core 0: sum the per-prefix contributions of all prefixes sharing i1 (contiguous)
  SegArgs a0 = {sh.S1, plan->counts + 1, plan->max_prefixes, plan->uniq_pref, sh.n2, nullptr,
                plan->i1_seg, plan->t1buf, strips, dcore[0], sh.S1, sh.n1, 1, plan->partial, TT_SEG_MIN_CHUNK, plan, -1};
  if ((st = seg_sum(a0, s)) != TT_OK) return st;
  // 3c. core 1: per-i2 accumulation over prefixes (done inside the matrix-core kernel)
  if (!mfma)
    hipLaunchKernelGGL(k_bwd_dg2,
                     dim3(sh.n2, tt_ceil_div(sh.S2, TT_BLOCK), tt_ceil_div(sh.R1, TT_DG2_RT)),
                     dim3(TT_BLOCK), 0, s, sh, t->core[0], plan->uniq_pref, plan->prefs_by_i2,
                     plan->i2_seg, plan->hbuf, dcore[1]);
  return tt_launch_status();
}

tt_status ttk_backward_naive(const TTShape &sh, const tt_table *t, const int64_t *indices,
                             const int64_t *offsets, int64_t nnz, int64_t num_bags,
                             const float *grad_out, float *const dcore[3], hipStream_t s) {
  for (int k = 0; k < 3; ++k) {
    const size_t len = core_len(sh, k);
    int blocks = tt_ceil_div((long long)len, TT_BLOCK * 4);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(TT_BLOCK), 0, s, dcore[k], len);
  }
  if (nnz > 0) {
    long long blocks = nnz < 65536 ? nnz : 65536;
    hipLaunchKernelGGL(k_bwd_naive, dim3((unsigned)blocks), dim3(TT_BLOCK), bwd_lds_bytes(sh), s,
                       sh, t->core[0], t->core[1], t->core[2], indices, offsets, (int)nnz,
                       (int)num_bags, grad_out, dcore[0], dcore[1], dcore[2]);
  }
  return tt_launch_status();
}

tt_status ttk_sgd(const TTShape &sh, const tt_table *t, const tt_plan *plan,
                  const float *const dcore[3], float lr, hipStream_t s) {
  if (plan) {
    TTProfScope prof(plan, TT_KERNEL_SGD, s);
    hipLaunchKernelGGL(k_sgd_touched, dim3(sh.n1 + sh.n2 + sh.n3), dim3(TT_BLOCK), 0, s, sh,
                       t->core[0], t->core[1], t->core[2], dcore[0], dcore[1], dcore[2],
                       plan->i1_seg, plan->i2_seg, plan->i3_seg, lr);
  } else {
    for (int k = 0; k < 3; ++k) {
      const size_t len = core_len(sh, k);
      int blocks = tt_ceil_div((long long)len, TT_BLOCK * 4);
      if (blocks > 4096) blocks = 4096;
      hipLaunchKernelGGL(k_sgd_dense, dim3(blocks), dim3(TT_BLOCK), 0, s, t->core[k], dcore[k], len,
                         lr);
    }
  }
  return tt_launch_status();
}
