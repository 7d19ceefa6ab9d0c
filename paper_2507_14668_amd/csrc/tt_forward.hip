// Forward pass of the TT embedding bag (paper Section III-B; batch-level reuse, Section III-C).
//
// Planned arm: one workgroup per distinct (i1,i2) prefix forms the prefix product
// P12 = G1[i1] x G2[i2] once in LDS and multiplies it with G3[i3] for every distinct row
// under that prefix; a second kernel sums the rows of each bag (gather-bound).
// Naive arm: one workgroup per bag runs the full three-slice chain for every lookup.
#include "tt_internal.h"

namespace {

// P12[j1][j2][r2] = sum_r1 G1[i1][j1][r1] * G2[r1][i2][j2][r2], written to LDS with row stride
// R2p over (j1,j2).  g1s must already hold the core-0 slice.  Consecutive threads take
// consecutive (j2,r2) so the core-1 reads are coalesced 4-byte streams of S2 floats per r1.
__device__ __forceinline__ void prefix_product(const TTShape &sh, const float *__restrict__ g2,
                                               int i2, const float *g1s, float *p12) {
  for (int o = threadIdx.x; o < sh.P; o += blockDim.x) {
    const int j1 = o / sh.S2, c = o - j1 * sh.S2;
    const float *col = g2 + (size_t)i2 * sh.S2 + c;
    float acc = 0.f;
    for (int r1 = 0; r1 < sh.R1; ++r1)
      acc = fmaf(g1s[j1 * sh.R1 + r1], col[(size_t)r1 * sh.n2 * sh.S2], acc);
    const int jj = j1 * sh.d2 + c / sh.R2, r2 = c % sh.R2;
    p12[jj * sh.R2p + r2] = acc;
  }
}

// row[(j1,j2)][j3] = sum_r2 P12[(j1,j2)][r2] * G3[r2][i3][j3] for output element o < D.
__device__ __forceinline__ float row_element(const TTShape &sh, const float *p12,
                                             const float *g3s, int o) {
  const int jj = o / sh.d3, j3 = o - jj * sh.d3;
  float acc = 0.f;
  for (int r2 = 0; r2 < sh.R2; ++r2) acc = fmaf(p12[jj * sh.R2p + r2], g3s[r2 * sh.d3 + j3], acc);
  return acc;
}

__device__ __forceinline__ void load_g3_slice(const TTShape &sh, const float *__restrict__ g3,
                                              int i3, float *g3s, int tid, int nthreads) {
  for (int e = tid; e < sh.S3; e += nthreads) {
    const int r2 = e / sh.d3, j3 = e - r2 * sh.d3;
    g3s[e] = g3[((size_t)r2 * sh.n3 + i3) * sh.d3 + j3];
  }
}

// LDS layout (floats): g1s[S1] | p12[d1*d2*R2p] | g3s[rows_per_iter * S3]
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_fwd_prefix_rows(TTArg<BATCHED> a, int rows_per_iter) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int32_t *__restrict__ counts = d.plan.counts, *__restrict__ uniq_pref = d.plan.uniq_pref,
                *__restrict__ pref_seg = d.plan.pref_seg, *__restrict__ uniq_row = d.plan.uniq_row;
  float *__restrict__ rowbuf = d.plan.rowbuf;
  extern __shared__ float lds[];
  float *g1s = lds, *p12 = g1s + sh.S1, *g3s = p12 + sh.d1 * sh.d2 * sh.R2p;
  const int up = counts[1];
  for (int q = blockIdx.x; q < up; q += gridDim.x) {
    const int p = uniq_pref[q], i1 = p / sh.n2, i2 = p - i1 * sh.n2;
    for (int e = threadIdx.x; e < sh.S1; e += blockDim.x) g1s[e] = g1[(size_t)i1 * sh.S1 + e];
    __syncthreads();
    prefix_product(sh, g2, i2, g1s, p12);
    __syncthreads();
    const int u0 = pref_seg[q], u1 = pref_seg[q + 1];
    // rows_per_iter rows at a time: thread group `sub` owns row u + sub
    const int sub = threadIdx.x / sh.D, tin = threadIdx.x - sub * sh.D;
    for (int u = u0; u < u1; u += rows_per_iter) {
      if (rows_per_iter == 1) {
        load_g3_slice(sh, g3, uniq_row[u] % sh.n3, g3s, threadIdx.x, blockDim.x);
      } else if (sub < rows_per_iter && u + sub < u1) {
        load_g3_slice(sh, g3, uniq_row[u + sub] % sh.n3, g3s + sub * sh.S3, tin, sh.D);
      }
      __syncthreads();
      if (rows_per_iter == 1) {
        for (int o = threadIdx.x; o < sh.D; o += blockDim.x)
          rowbuf[(size_t)u * sh.D + o] = row_element(sh, p12, g3s, o);
      } else if (sub < rows_per_iter && u + sub < u1) {
        rowbuf[(size_t)(u + sub) * sh.D + tin] = row_element(sh, p12, g3s + sub * sh.S3, tin);
      }
      __syncthreads();
    }
  }
}

#define TT_BAG_BLOCK 64

// VEC consecutive columns of distinct row u (zeros for an invalid lookup, u < 0).
template <int VEC>
__device__ __forceinline__ void load_row_vec(const float *__restrict__ rowbuf, int u, int D, int c,
                                             float (&x)[VEC]) {
  if (u < 0) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = 0.f;
  } else if (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4 *>(rowbuf + (size_t)u * D + c);
    x[0] = t.x; x[1 % VEC] = t.y; x[2 % VEC] = t.z; x[3 % VEC] = t.w;
  } else {
    x[0] = rowbuf[(size_t)u * D + c];
  }
}

// out[b][:] = sum over the lookups of bag b of rowbuf[lookup2row[l]][:].
// A group of LANES lanes owns one bag; each lane owns VEC consecutive columns per step.
template <bool BATCHED, int VEC>
__global__ void __launch_bounds__(TT_BLOCK)
k_bag_sum(TTArg<BATCHED> a, int lanes) {
  const TTDev &d = a.get();
  const int D = d.sh.D, num_bags = d.num_bags, nnz = d.nnz;
  const int64_t *__restrict__ offsets = d.offsets;
  const int32_t *__restrict__ lookup2row = d.plan.lookup2row;
  const float *__restrict__ rowbuf = d.plan.rowbuf;
  float *__restrict__ out = d.out;
  const int groups_per_block = blockDim.x / lanes;
  const int g = threadIdx.x / lanes, lane = threadIdx.x - g * lanes;
  const int stride = gridDim.x * groups_per_block;
  int b = blockIdx.x * groups_per_block + g;
  // One-lookup bags (one-hot features), four bags of a lane group at a time: the four chains
  // offsets -> row slot -> row -> store are independent and overlap.  Same arithmetic as the general
  // path below (0 + row), so the result does not depend on which path served a bag.
  for (; b + 3 * stride < num_bags; b += 4 * stride) {
    long long o[4][2];
#pragma unroll
    for (int k = 0; k < 4; ++k) { o[k][0] = offsets[b + k * stride]; o[k][1] = offsets[b + k * stride + 1]; }
    bool single = true;
#pragma unroll
    for (int k = 0; k < 4; ++k) single = single && o[k][0] >= 0 && o[k][0] < nnz && o[k][1] == o[k][0] + 1;
    if (!single) break;  // the general path takes over from bag b (the same for every lane of the group)
    int u[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) u[k] = lookup2row[o[k][0]];
    for (int c = lane * VEC; c < D; c += lanes * VEC) {
      float x[4][VEC];
#pragma unroll
      for (int k = 0; k < 4; ++k) load_row_vec<VEC>(rowbuf, u[k], D, c, x[k]);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float t[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) t[v] = 0.f + (0.f + x[k][v]);
        float *dst = out + (size_t)(b + k * stride) * D + c;
        if (VEC == 4) tt_store_stream4(dst, t[0], t[1 % VEC], t[2 % VEC], t[3 % VEC]);
        else dst[0] = t[0];
      }
    }
  }
  for (; b < num_bags; b += stride) {
    // offsets are clamped to [0, nnz] so that a malformed CSR array cannot index out of bounds
    const long long o0 = offsets[b], o1 = offsets[b + 1];
    const int l0 = o0 < 0 ? 0 : (o0 > nnz ? nnz : (int)o0), l1 = o1 < l0 ? l0 : (o1 > nnz ? nnz : (int)o1);
    for (int c = lane * VEC; c < D; c += lanes * VEC) {
      // two-level sum: blocks of TT_BAG_BLOCK lookups are summed first and then added to the
      // running total, so rounding error grows with len/TT_BAG_BLOCK instead of len
      float tot[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) tot[v] = 0.f;
      for (int base = l0; base < l1; base += TT_BAG_BLOCK) {
        const int stop = base + TT_BAG_BLOCK < l1 ? base + TT_BAG_BLOCK : l1;
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        int l = base;
        for (; l + 4 <= stop; l += 4) {  // four independent gathers in flight
          int u[4];
          float x[4][VEC];
#pragma unroll
          for (int k = 0; k < 4; ++k) u[k] = lookup2row[l + k];
#pragma unroll
          for (int k = 0; k < 4; ++k) load_row_vec<VEC>(rowbuf, u[k], D, c, x[k]);
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] += (x[0][v] + x[1][v]) + (x[2][v] + x[3][v]);
        }
        for (; l < stop; ++l) {
          float x[VEC];
          load_row_vec<VEC>(rowbuf, lookup2row[l], D, c, x);
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] += x[v];
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) tot[v] += acc[v];
      }
      if (VEC == 4) {
        tt_store_stream4(out + (size_t)b * D + c, tot[0], tot[1 % VEC], tot[2 % VEC], tot[3 % VEC]);
      } else {
        out[(size_t)b * D + c] = tot[0];
      }
    }
  }
}

// Naive arm: workgroup per bag; every lookup recomputes its prefix product and row.
// LDS layout: g1s[S1] | p12[d1*d2*R2p] | g3s[S3]
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_fwd_naive(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int64_t *__restrict__ indices = d.indices, *__restrict__ offsets = d.offsets;
  const int num_bags = d.num_bags, nnz = d.nnz;
  float *__restrict__ out = d.out;
  extern __shared__ float lds[];
  float *g1s = lds, *p12 = g1s + sh.S1, *g3s = p12 + sh.d1 * sh.d2 * sh.R2p;
  constexpr int MAXO = 4;  // D <= 1024 columns over 256 threads
  for (int b = blockIdx.x; b < num_bags; b += gridDim.x) {
    float acc[MAXO], tot[MAXO];
#pragma unroll
    for (int k = 0; k < MAXO; ++k) acc[k] = tot[k] = 0.f;
    long long l0 = offsets[b], l1 = offsets[b + 1];  // clamped: malformed offsets stay in bounds
    l0 = l0 < 0 ? 0 : (l0 > nnz ? nnz : l0);
    l1 = l1 < l0 ? l0 : (l1 > nnz ? nnz : l1);
    for (long long l = l0; l < l1; ++l) {
      const long long row = indices[l];
      if (((l - l0) % TT_BAG_BLOCK) == 0) {  // two-level sum as in the planned arm
#pragma unroll
        for (int k = 0; k < MAXO; ++k) { tot[k] += acc[k]; acc[k] = 0.f; }
      }
      if (row < 0 || row >= sh.num_rows) continue;  // uniform across the workgroup
      const int i3 = (int)(row % sh.n3), p = (int)(row / sh.n3), i1 = p / sh.n2,
                i2 = p - i1 * sh.n2;
      for (int e = threadIdx.x; e < sh.S1; e += blockDim.x) g1s[e] = g1[(size_t)i1 * sh.S1 + e];
      load_g3_slice(sh, g3, i3, g3s, threadIdx.x, blockDim.x);
      __syncthreads();
      prefix_product(sh, g2, i2, g1s, p12);
      __syncthreads();
#pragma unroll
      for (int k = 0; k < MAXO; ++k) {
        const int o = threadIdx.x + k * TT_BLOCK;
        if (o < sh.D) acc[k] += row_element(sh, p12, g3s, o);
      }
      __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < MAXO; ++k) {
      const int o = threadIdx.x + k * TT_BLOCK;
      if (o < sh.D) out[(size_t)b * sh.D + o] = tot[k] + acc[k];
    }
  }
}

size_t fwd_lds_bytes(const TTShape &sh, int rows_per_iter) {
  return sizeof(float) * ((size_t)sh.S1 + (size_t)sh.d1 * sh.d2 * sh.R2p +
                          (size_t)rows_per_iter * sh.S3);
}

}  // namespace

tt_status ttk_forward_plan(const TTBatch &b, hipStream_t s) {
  const TTShape &sh = b.host[0].sh;  // d[] and r[] are common to the batch
  const long long max_pref = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_prefixes; });
  if (max_pref > 0 && ttk_batch_mfma(b)) {
    tt_status st = ttk_forward_mfma(b, s);
    if (st != TT_OK) return st;
  } else if (max_pref > 0) {
    int rows_per_iter = TT_BLOCK / sh.D;
    if (rows_per_iter < 1) rows_per_iter = 1;
    if (rows_per_iter > 8) rows_per_iter = 8;
    const long long blocks = max_pref < 4096 ? max_pref : 4096;
    TTProfScope prof(&b.host[0].plan, TT_KERNEL_FWD_CONTRACT, s);
    TT_LAUNCH(k_fwd_prefix_rows, blocks, TT_BLOCK, fwd_lds_bytes(sh, rows_per_iter), s, b, rows_per_iter);
  }
  return ttk_bag_sum(b, s);
}

tt_status ttk_bag_sum(const TTBatch &b, hipStream_t s) {
  const TTShape &sh = b.host[0].sh;
  const long long max_bags = tt_batch_max(b, [](const TTDev &d) { return (long long)d.num_bags; });
  if (max_bags > 0) {
    bool vec4 = (sh.D % 4) == 0;
    for (int t = 0; t < b.T; ++t) vec4 = vec4 && ((uintptr_t)b.host[t].out % 16) == 0;
    int lanes = 1;
    while (lanes < TT_WAVE && lanes * (vec4 ? 4 : 1) < sh.D) lanes <<= 1;
    const int groups = TT_BLOCK / lanes;
    long long blocks = (max_bags + groups - 1) / groups;
    // a batch of one-lookup bags (as many lookups as bags) lets every lane group take four bags at a time
    bool one_hot = true;
    for (int t = 0; t < b.T; ++t) one_hot = one_hot && b.host[t].nnz == b.host[t].num_bags;
    if (one_hot) blocks = (blocks + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    TTProfScope prof(&b.host[0].plan, TT_KERNEL_BAG_SUM, s);
    if (vec4) TT_LAUNCH_T(k_bag_sum, 4, blocks, TT_BLOCK, 0, s, b, lanes);
    else TT_LAUNCH_T(k_bag_sum, 1, blocks, TT_BLOCK, 0, s, b, lanes);
  }
  return tt_launch_status();
}

tt_status ttk_forward_naive(const TTBatch &b, hipStream_t s) {
  const long long max_bags = tt_batch_max(b, [](const TTDev &d) { return (long long)d.num_bags; });
  if (max_bags == 0) return TT_OK;
  const long long blocks = max_bags < 65536 ? max_bags : 65536;
  TT_LAUNCH(k_fwd_naive, blocks, TT_BLOCK, fwd_lds_bytes(b.host[0].sh, 1), s, b);
  return tt_launch_status();
}
