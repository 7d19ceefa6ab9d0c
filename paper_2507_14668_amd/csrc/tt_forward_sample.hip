// Sample-level reuse forward of the TT embedding bag (paper Section III-B, reuse equation: lookups
// of one bag that share the first two TT indices run one product chain whose third factor is the sum
// of their core-2 slices) on top of the batch-level reuse buffer (Section III-C: one product
// G1[i1] x G2[i2] per distinct prefix of the batch, kept in device memory).
//
//   k_p12_fill   reuse buffer: P12[q][(j1,j2)][r2] for every distinct prefix q of the batch (tables
//                the matrix-core kernels serve fill it with the forward contraction kernel instead)
//   k_bag_chains one wavefront per bag: the bag's lookups are grouped by prefix slot (wavefront
//                ballots, no sorting), each group sums its core-2 slices into S[r2][j3] and adds
//                P12[q] x S to the bag's row, which is written once.  No atomics, no row buffer, no
//                separate bag-sum launch; the price is one read of a whole prefix product per
//                (bag, prefix) group instead of one read of a finished row per lookup.
#include "tt_internal.h"

namespace {

template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_p12_fill(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1];
  const int32_t *__restrict__ counts = d.plan.counts, *__restrict__ uniq_pref = d.plan.uniq_pref;
  float *__restrict__ p12buf = d.p12buf;
  extern __shared__ float lds[];
  float *g1s = lds;  // [d1][R1]
  const int up = counts[1];
  for (int q = blockIdx.x; q < up; q += gridDim.x) {
    const int p = uniq_pref[q], i1 = p / sh.n2, i2 = p - i1 * sh.n2;
    __syncthreads();  // the previous prefix's readers of g1s are done
    for (int e = threadIdx.x; e < sh.S1; e += blockDim.x) g1s[e] = g1[(size_t)i1 * sh.S1 + e];
    __syncthreads();
    // consecutive threads take consecutive (j2, r2): coalesced reads of core 1 and writes of P12
    for (int o = threadIdx.x; o < sh.P; o += blockDim.x) {
      const int j1 = o / sh.S2, c = o - j1 * sh.S2;
      const float *col = g2 + (size_t)i2 * sh.S2 + c;
      float acc = 0.f;
      for (int r1 = 0; r1 < sh.R1; ++r1)
        acc = fmaf(g1s[j1 * sh.R1 + r1], col[(size_t)r1 * sh.n2 * sh.S2], acc);
      p12buf[(size_t)q * sh.P + o] = acc;  // o = (j1*d2 + j2)*R2 + r2
    }
  }
}

// NO = outputs per lane (D <= 64 * NO).  LDS per wavefront: the group's prefix product with row
// stride R2 + 1 (lanes of different (j1,j2) on different banks) and the slice sum S[r2][j3].
template <bool BATCHED, int NO>
__global__ void __launch_bounds__(TT_BLOCK)
k_bag_chains(TTArg<BATCHED> a, int lds_per_wave) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g3 = d.g[2];
  const float *__restrict__ p12buf = d.p12buf;
  const int64_t *__restrict__ offsets = d.offsets;
  const int32_t *__restrict__ lookup2row = d.plan.lookup2row, *__restrict__ row2pref = d.plan.row2pref,
                *__restrict__ uniq_row = d.plan.uniq_row;
  extern __shared__ float lds[];
  const int lane = threadIdx.x & (TT_WAVE - 1), wave = threadIdx.x / TT_WAVE;
  const int b = blockIdx.x * (blockDim.x / TT_WAVE) + wave;
  if (b >= d.num_bags) return;  // uniform for the wavefront; the kernel has no workgroup barrier
  float *Pw = lds + (size_t)wave * lds_per_wave, *Sw = Pw + sh.d1 * sh.d2 * (sh.R2 + 1);
  const int Rp = sh.R2 + 1;

  int prow[NO], scol[NO];
  float acc[NO];
#pragma unroll
  for (int k = 0; k < NO; ++k) {
    const int o = lane + TT_WAVE * k, jj = o / sh.d3;
    prow[k] = (o < sh.D ? jj : 0) * Rp;
    scol[k] = o < sh.D ? o - jj * sh.d3 : 0;
    acc[k] = 0.f;
  }
  // offsets are clamped to [0, nnz] so that a malformed CSR array cannot index out of bounds
  const long long o0 = offsets[b], o1 = offsets[b + 1], nnz = d.nnz;
  const long long lo = o0 < 0 ? 0 : (o0 > nnz ? nnz : o0), hi = o1 < lo ? lo : (o1 > nnz ? nnz : o1);
  const bool vec4 = (sh.R2 & 3) == 0;  // the buffer is 256-byte aligned and P a multiple of 4 then
  for (long long base = lo; base < hi; base += TT_WAVE) {
    // this lane's lookup: prefix slot and i3 (an invalid lookup has no row slot and takes no part)
    const long long l = base + lane;
    const int u = l < hi ? lookup2row[l] : -1;
    const int q = u >= 0 ? row2pref[u] : -1;
    const int i3 = u >= 0 ? uniq_row[u] - tt_div(uniq_row[u], sh.mul3, sh.sh3) * sh.n3 : 0;
    unsigned long long left = __ballot(q >= 0);
    while (left) {  // uniform: one round per distinct prefix among the 64 lookups
      const int first = __ffsll(left) - 1;
      const int qg = __builtin_amdgcn_readlane(q, first);
      const unsigned long long members = __ballot(q == qg);
      left &= ~members;
      // the group's prefix product: device memory -> LDS
      const float *src = p12buf + (size_t)qg * sh.P;
      if (vec4) {
        for (int e = lane * 4; e < sh.P; e += TT_WAVE * 4) {
          const float4 v = *reinterpret_cast<const float4 *>(src + e);
          const int row = e / sh.R2, c = e - row * sh.R2;
          float *dst = Pw + row * Rp + c;
          dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
      } else {
        for (int e = lane; e < sh.P; e += TT_WAVE) {
          const int row = e / sh.R2;
          Pw[row * Rp + (e - row * sh.R2)] = src[e];
        }
      }
      // S[r2][j3] = sum over the group's lookups, in bag order, of G3[r2][i3][j3]; four lookups per
      // round so that their loads are issued together
      for (int e0 = 0; e0 < sh.S3; e0 += TT_WAVE) {  // uniform trip count: every lane reaches the lane reads
        const int e = e0 + lane < sh.S3 ? e0 + lane : 0, r2 = e / sh.d3, j3 = e - r2 * sh.d3;
        const float *gp = g3 + (size_t)r2 * sh.n3 * sh.d3 + j3;
        float sum = 0.f;
        unsigned long long mm = members;
        while (mm) {
          float v[4];
          bool has[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            has[j] = mm != 0;
            const int m = has[j] ? __ffsll(mm) - 1 : first;
            mm &= mm - 1;  // stays 0 once it is 0
            v[j] = gp[(size_t)__builtin_amdgcn_readlane(i3, m) * sh.d3];
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) sum += has[j] ? v[j] : 0.f;
        }
        if (e0 + lane < sh.S3) Sw[e] = sum;
      }
      tt_wave_lds_order();
#pragma unroll 4
      for (int r2 = 0; r2 < sh.R2; ++r2) {
#pragma unroll
        for (int k = 0; k < NO; ++k) acc[k] = fmaf(Pw[prow[k] + r2], Sw[r2 * sh.d3 + scol[k]], acc[k]);
      }
      tt_wave_lds_order();  // the next group overwrites Pw and Sw
    }
  }
#pragma unroll
  for (int k = 0; k < NO; ++k) {
    const int o = lane + TT_WAVE * k;
    if (o < sh.D) d.out[(size_t)b * sh.D + o] = acc[k];
  }
}

}  // namespace

size_t ttk_bag_chains_lds_per_wave(const TTShape &sh) {
  return (size_t)sh.d1 * sh.d2 * (sh.R2 + 1) + sh.S3;
}

tt_status ttk_forward_sample(const TTBatch &b, hipStream_t s) {
  const TTShape &sh = b.host[0].sh;
  // reuse buffer
  if (ttk_batch_mfma(b)) {
    tt_status st = ttk_forward_mfma_p12(b, s);
    if (st != TT_OK) return st;
  } else {
    const long long cap = tt_batch_max(b, [](const TTDev &d) { return (long long)d.plan.max_prefixes; });
    const int grid = (int)(cap < 1 ? 1 : (cap > 8192 ? 8192 : cap));
    TTProfScope prof(&b.host[0].plan, TT_KERNEL_P12_FILL, s);
    TT_LAUNCH(k_p12_fill, grid, TT_BLOCK, sh.S1 * sizeof(float), s, b);
    if (tt_launch_status() != TT_OK) return TT_ERR_HIP;
  }
  // bags: as many wavefronts per workgroup (4, 2 or 1) as fit in 64 KB of LDS
  const size_t per_wave = ttk_bag_chains_lds_per_wave(sh);
  int waves = 4;
  while (waves > 1 && waves * per_wave * sizeof(float) > 65536) waves >>= 1;
  if (waves * per_wave * sizeof(float) > 65536) return TT_ERR_SHAPE;
  const long long bags = tt_batch_max(b, [](const TTDev &d) { return (long long)d.num_bags; });
  if (bags == 0) return TT_OK;
  const int grid = tt_ceil_div(bags, waves);
  const size_t lds = waves * per_wave * sizeof(float);
  const int no = tt_ceil_div(sh.D, TT_WAVE);
  TTProfScope prof(&b.host[0].plan, TT_KERNEL_BAG_CHAINS, s);
  if (no <= 1) TT_LAUNCH_T(k_bag_chains, 1, grid, waves * TT_WAVE, lds, s, b, (int)per_wave);
  else if (no <= 2) TT_LAUNCH_T(k_bag_chains, 2, grid, waves * TT_WAVE, lds, s, b, (int)per_wave);
  else if (no <= 4) TT_LAUNCH_T(k_bag_chains, 4, grid, waves * TT_WAVE, lds, s, b, (int)per_wave);
  else if (no <= 8) TT_LAUNCH_T(k_bag_chains, 8, grid, waves * TT_WAVE, lds, s, b, (int)per_wave);
  else TT_LAUNCH_T(k_bag_chains, 16, grid, waves * TT_WAVE, lds, s, b, (int)per_wave);
  return tt_launch_status();
}
