// MFMA forward contraction for the TT embedding bag (paper Section III-B/III-C), gfx950.
//
// Work is grouped by i2: one workgroup owns one (i2, 256-column strip of the core-1 slice
// G2[:, i2, :, :]) -- the strip is a range of j2, all r2, so that a strip yields complete output
// columns -- keeps the strip in registers, and walks the distinct prefixes (i1, i2) of the batch in
// chunks of TT_MP = 8.  For a chunk
//   F1: P12[(p,j1)][(j2,r2)] = sum_r1 G1[i1_p][j1][r1] * G2[r1][i2][j2][r2]
// is a 32 x R1 x 256 GEMM on v_mfma_f32_16x16x4_f32 (A = the 8 core-0 slices staged in LDS,
// B = the strip), so every core-1 element is loaded from memory once per workgroup and feeds all
// prefixes of its i2.  The product is written to LDS and
//   F2: row[(j1,j2)][j3] = sum_r2 P12[(j1,j2)][r2] * G3[r2][i3][j3]
// runs per (prefix, four distinct rows) as a 16 x R2 x (4*JW) MFMA GEMM whose A operand is
// gathered from core 2; rows are stored as float4.
//
// A workgroup has eight wavefronts (32 strip columns each in F1; the row quads of F2 are dealt
// round-robin) and 45 KB of LDS, so two workgroups = four wavefronts per SIMD share a compute unit
// and cover each other's memory waits.  Tables with few core-1 slices deal the chunks of one
// (i2, strip) to several workgroups (each loads the strip; the outputs are per row, so nothing has
// to be combined).
//
// Operand layout of __builtin_amdgcn_mfma_f32_16x16x4f32 (D = A[16x4] * B[4x16] + C):
//   lane l supplies A[m = l%16][k = l/16] and B[k = l/16][n = l%16];
//   lane l holds C[m = 4*(l/16) + v][n = l%16] in component v of its float4.
#include <mutex>

#include "tt_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short bf16x4 __attribute__((ext_vector_type(4)));  // four bf16 values as the 16x16x16 MFMA takes them

__device__ __forceinline__ float bf16_to_float(unsigned short v) { return __uint_as_float((unsigned)v << 16); }

constexpr int FTHR = 512;   // threads per workgroup
#ifndef TT_FWD_WG_TARGET
#define TT_FWD_WG_TARGET 512   // workgroups a launch should have at least (two per compute unit)
#endif
#define TT_FWD_MAX_SPLIT 16
constexpr int FMETA = 64;   // prefixes whose plan entries are fetched into LDS in one go (8 chunks)
constexpr int FWD_I3_STAGE = FTHR / TT_MP;  // i3 of the first 64 distinct rows of each prefix is staged in LDS

template <int R1, int R2, int D2>
struct FwdGeom {
  static constexpr int JW = 256 / R2;      // j2 values covered by one 256-column strip
  static constexpr int NSTRIP = D2 / JW;   // strips per i2
  static constexpr int S2 = D2 * R2;       // floats per r1-chunk of a core-1 slice
  static constexpr int CC = 4 * JW;        // (j1, j2) columns per strip
  // LDS strides: a 64-lane access is served in two halves (lanes 0-31: lq = 0,1); each stride puts
  // the 32 lanes of a half on 32 different banks
  static constexpr int RS = R1 + 2;        // core-0 tile [32 (p,j1)][R1]: F1 A operand, row = lm, + lq
  static constexpr int Rp = R2 + 2;        // P12 row [(j1,j2)][r2]: F2 B operand, row = lm, + lq
  static constexpr int PS = CC * Rp + 1;   // P12 block of a prefix: F1 store, even banks for lq = 0, odd for lq = 1
  static constexpr int KS1 = R1 / 4, KS2 = R2 / 4;
  static constexpr int NT2 = CC / 16;
  static constexpr int D = 4 * D2 * 4, S1 = 4 * R1;
  static constexpr int OFF_P12 = 32 * RS;
  static constexpr size_t LDS_FLOATS = (size_t)OFF_P12 + TT_MP * PS;
  static constexpr int GPT = (32 * R1) / FTHR;  // core-0 tile elements per thread
  static_assert(256 % R2 == 0 && D2 % JW == 0 && R1 % 16 == 0 && CC % 16 == 0 && TT_MP == 8, "unsupported shape");
};

// P12OUT: the kernel stops after F1 and stores the prefix products to the reuse buffer
// [prefix slot][(j1,j2)][r2] instead of running F2 (first stage of the sample-level forward).
// BF16: the cores are bf16 copies made by k_cores_to_bf16 (cores 0 and 2 in their own layout, core 1
// as [i2][r1 / 4][(j2, r2)][r1 % 4] so that a lane's four consecutive r1 of one column are 8
// contiguous bytes).  F1 runs on v_mfma_f32_16x16x16_bf16 (lane l supplies A[m = l%16][k = 4*(l/16) + i]
// and B[k = 4*(l/16) + i][n = l%16], i = 0..3; C as for 16x16x4) with fp32 accumulators, the products
// stay fp32 in LDS, and F2 is the fp32 MFMA with core-2 values widened exactly: the only difference
// from the fp32 path is the rounding of the stored cores.
template <bool BATCHED, int R1, int R2, int D2, bool P12OUT, bool BF16>
__global__ void __launch_bounds__(FTHR, 4)  // four wavefronts per SIMD: two workgroups per compute unit
k_fwd_mfma(TTArg<BATCHED> a, int split) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int32_t *__restrict__ uniq_row = d.plan.uniq_row, *__restrict__ i2_seg = d.plan.i2_seg;
  const int4 *__restrict__ pref_meta = reinterpret_cast<const int4 *>(d.plan.pref_meta);
  float *__restrict__ rowbuf = d.plan.rowbuf, *__restrict__ p12buf = d.p12buf;
  using G = FwdGeom<R1, R2, D2>;
  extern __shared__ float lds[];
  float *As = lds;                  // [32][RS]  core-0 slices of the chunk
  unsigned short *Asb = reinterpret_cast<unsigned short *>(lds);  // BF16: the same tile as [32][R1 + 4] bf16
  constexpr int RSB = R1 + 4;
  const unsigned short *__restrict__ g1b = reinterpret_cast<const unsigned short *>(d.g[0]),
                       *__restrict__ g2b = reinterpret_cast<const unsigned short *>(d.g[1]),
                       *__restrict__ g3b = reinterpret_cast<const unsigned short *>(d.g[2]);
  float *P12s = lds + G::OFF_P12;   // [8][PS]   prefix products of the chunk
  __shared__ int s_i1[FMETA], s_u0[FMETA], s_nr[FMETA], s_slot[FMETA];
  __shared__ int s_item_off[2][TT_MP + 1];
  __shared__ int s_i3[2][TT_MP][FWD_I3_STAGE];

  // Workgroup index = ((i2 / 8) * (strips * split) + (strip, part)) * 8 + i2 % 8: workgroups are
  // dealt to the 8 XCDs round-robin, so all strips and parts of one i2 run on XCD i2 % 8, close in
  // time (they read the same core-0 slices, plan entries and core-2 rows).
  const int nsub = G::NSTRIP * split;
  const int i2 = (int)(blockIdx.x / (8 * nsub)) * 8 + (int)(blockIdx.x & 7), sub = (int)(blockIdx.x >> 3) % nsub;
  if (i2 >= sh.n2) return;  // padding of the last group of 8, or a table of the batch with fewer i2 values
  const int strip = sub / split, part = sub - strip * split;
  const int j2base = strip * G::JW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lm = lane & 15, lq = lane >> 4;

  // This wavefront's 32 columns of the strip of G2[:, i2], all r1 (B operand of F1), as one float2
  // per row and lane: lane lm holds columns 2*lm, 2*lm + 1, and MFMA tile nt takes component nt, i.e.
  // tile column lm stands for strip column 32*wave + 2*lm + nt.  Requested before the plan is looked at.
  float2 bq[BF16 ? 1 : G::KS1];
  uint4 bqb[BF16 ? R1 / 16 : 1];  // BF16: per 16 values of r1, columns 2*lm and 2*lm + 1 with four r1 each
  if constexpr (BF16) {
#pragma unroll
    for (int ks = 0; ks < R1 / 16; ++ks)
      bqb[ks] = *reinterpret_cast<const uint4 *>(g2b + (((size_t)i2 * (R1 / 4) + 4 * ks + lq) * G::S2 + strip * 256 +
                                                        32 * wave + 2 * lm) * 4);
  } else {
#pragma unroll
    for (int ks = 0; ks < G::KS1; ++ks)
      bq[ks] = *reinterpret_cast<const float2 *>(g2 + ((size_t)(4 * ks + lq) * sh.n2 + i2) * G::S2 + strip * 256 +
                                                 32 * wave + 2 * lm);
  }

  int seg0 = i2_seg[i2], seg1 = i2_seg[i2 + 1];
  if (split > 1) {  // the chunks of this (i2, strip) are dealt in contiguous runs to `split` workgroups
    const int nch = (seg1 - seg0 + TT_MP - 1) / TT_MP, per = (nch + split - 1) / split;
    const int c0 = part * per, c1 = (c0 + per) < nch ? (c0 + per) : nch;
    const int lo = seg0 + c0 * TT_MP, hi = seg0 + c1 * TT_MP;
    seg1 = c0 < c1 ? (hi < seg1 ? hi : seg1) : seg0;
    seg0 = c0 < c1 ? lo : seg0;
  }
  if (seg0 == seg1) return;  // uniform: no prefix for this workgroup

  // Global-memory operands of the NEXT chunk (core-0 rows, row ids of its first rows) are fetched
  // into registers while the current chunk computes.
  float g1n[G::GPT];
  int rown = 0;
  auto fetch_meta = [&](int base) __attribute__((always_inline)) {  // plan entries of prefixes base .. base+63 -> LDS
    if (threadIdx.x < FMETA) {
      int i1 = -1, u0 = 0, nr = 0, slot = 0;
      if (base + (int)threadIdx.x < seg1) {
        const int4 m = pref_meta[base + threadIdx.x];  // i1, first row slot, rows, prefix slot
        i1 = m.x; u0 = m.y; nr = m.z; slot = m.w;
      }
      s_i1[threadIdx.x] = i1; s_u0[threadIdx.x] = u0; s_nr[threadIdx.x] = nr; s_slot[threadIdx.x] = slot;
    }
  };
  auto fetch_chunk = [&](int mo) __attribute__((always_inline)) {  // mo = offset of the chunk inside the staged plan entries
#pragma unroll
    for (int k = 0; k < G::GPT; ++k) {
      const int e = threadIdx.x + k * FTHR, row = e / R1, r1 = e - row * R1;
      // unconditional (slice 0 stands in for a prefix the chunk does not have; it is replaced by
      // zero when the chunk is staged, so that no load sits under a branch)
      const int i1 = s_i1[mo + (row >> 2)];
      const size_t at = (size_t)(i1 >= 0 ? i1 : 0) * G::S1 + (row & 3) * R1 + r1;
      g1n[k] = BF16 ? bf16_to_float(g1b[at]) : g1[at];
    }
    const int p = threadIdx.x / FWD_I3_STAGE, r = threadIdx.x - p * FWD_I3_STAGE;
    rown = uniq_row[s_u0[mo + p] + (r < s_nr[mo + p] ? r : 0)];
  };
  auto stage_chunk = [&](int par, int mo) __attribute__((always_inline)) {  // registers -> LDS
#pragma unroll
    for (int k = 0; k < G::GPT; ++k) {
      const int e = threadIdx.x + k * FTHR, row = e / R1, r1 = e - row * R1;
      const float v = s_i1[mo + (row >> 2)] >= 0 ? g1n[k] : 0.f;  // zero rows for prefixes the chunk does not have
      if constexpr (BF16) Asb[row * RSB + r1] = (unsigned short)(__float_as_uint(v) >> 16);  // exact: v is a bf16 value
      else As[row * G::RS + r1] = v;
    }
    s_i3[par][threadIdx.x / FWD_I3_STAGE][threadIdx.x % FWD_I3_STAGE] = rown % sh.n3;
    if (wave == 0) {  // quads per prefix of the chunk, running total (scan over the first 8 lanes)
      const int q4 = lane < TT_MP ? (s_nr[mo + lane] + 3) >> 2 : 0;
      int incl = q4;
#pragma unroll
      for (int o = 1; o < TT_MP; o <<= 1) {
        const int t = __shfl_up(incl, o, TT_WAVE);
        if (lane >= o) incl += t;
      }
      if (lane < TT_MP) s_item_off[par][lane] = incl - q4;
      if (lane == TT_MP - 1) s_item_off[par][TT_MP] = incl;
    }
  };

  fetch_meta(seg0);
  __syncthreads();
  fetch_chunk(0);
  stage_chunk(0, 0);
  int par = 0;

  for (int cs = seg0; cs < seg1; cs += TT_MP) {
    const int mo = (cs - seg0) % FMETA;  // this chunk's offset in s_i1 / s_u0 / s_nr
    const bool more = cs + TT_MP < seg1, refill = mo + TT_MP == FMETA;
    __syncthreads();  // this chunk's staging is visible; the previous chunk's readers of P12 are done
    if (more && !refill) fetch_chunk(mo + TT_MP);  // next chunk's operands, staged after F1

    // ---- F1: C[32 x 32 per wavefront] on MFMA -> P12s[p][(j1, j2)][r2] ---------------------------
    {
      f32x4 acc[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if constexpr (BF16) {
#pragma unroll
        for (int ks = 0; ks < R1 / 16; ++ks) {
          bf16x4 av[2], bv[2];
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            av[mt] = *reinterpret_cast<const bf16x4 *>(Asb + (16 * mt + lm) * RSB + 16 * ks + 4 * lq);
          const uint2 b0 = make_uint2(bqb[ks].x, bqb[ks].y), b1 = make_uint2(bqb[ks].z, bqb[ks].w);
          bv[0] = *reinterpret_cast<const bf16x4 *>(&b0);
          bv[1] = *reinterpret_cast<const bf16x4 *>(&b1);
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av[mt], bv[nt], acc[mt][nt], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < G::KS1; ++ks) {
          float av[2];
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) av[mt] = As[(16 * mt + lm) * G::RS + 4 * ks + lq];
          const float bv[2] = {bq[ks].x, bq[ks].y};
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mt], bv[nt], acc[mt][nt], 0, 0, 0);
        }
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int p = 4 * mt + lq;  // C row m = 4*lq + v  ->  prefix 4*mt + lq, j1 = v
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const int cl = 32 * wave + 2 * lm + nt, j2loc = cl / R2, r2 = cl - j2loc * R2;
#pragma unroll
          for (int v = 0; v < 4; ++v)
            P12s[p * G::PS + (v * G::JW + j2loc) * G::Rp + r2] = acc[mt][nt][v];
        }
      }
    }
    __syncthreads();  // P12 of the chunk is complete; the core-0 tile is free
    if (more && !refill) stage_chunk(par ^ 1, mo + TT_MP);

    if constexpr (P12OUT) {  // the chunk's products -> reuse buffer, as float4 along r2
      constexpr int Q4 = G::CC * R2 / 4;  // float4 per prefix and strip
      for (int e = threadIdx.x; e < TT_MP * Q4; e += FTHR) {
        const int p = e / Q4, rem = e - p * Q4, cc = rem / (R2 / 4), r4 = rem - cc * (R2 / 4);
        if (s_i1[mo + p] < 0) continue;
        const int j1 = cc / G::JW, j2 = j2base + (cc - j1 * G::JW);
        const float *src = P12s + p * G::PS + cc * G::Rp + 4 * r4;
        *reinterpret_cast<float4 *>(p12buf + (size_t)s_slot[mo + p] * (4 * D2 * R2) + (j1 * D2 + j2) * R2 + 4 * r4) =
            make_float4(src[0], src[1], src[2], src[3]);
      }
    }
    // ---- F2: items = (prefix, four distinct rows), dealt round-robin to the wavefronts -------
    const int total = P12OUT ? 0 : s_item_off[par][TT_MP];
    struct Item { int p, ubase, nrow; float a[G::KS2]; };
    auto fetch = [&](int it, Item &x) __attribute__((always_inline)) {
      int p = 0;
#pragma unroll
      for (int k = 1; k < TT_MP; ++k) p += (s_item_off[par][k] <= it) ? 1 : 0;
      // p = number of k in 1..TT_MP-1 with item_off[k] <= it = the prefix whose range holds `it`
      const int quad = it - s_item_off[par][p];
      x.p = p;
      x.ubase = s_u0[mo + p] + 4 * quad;
      const int left = s_nr[mo + p] - 4 * quad;
      x.nrow = left < 4 ? left : 4;
      // A operand: G3[r2][i3(row)][j3], m = (row, j3) = lm, k = r2
      const int arow = 4 * quad + ((lm >> 2) < x.nrow ? (lm >> 2) : x.nrow - 1);
      const int i3 = arow < FWD_I3_STAGE ? s_i3[par][p][arow] : uniq_row[s_u0[mo + p] + arow] % sh.n3;
      const size_t a0 = ((size_t)lq * sh.n3 + i3) * 4 + (lm & 3);  // G3[r2 = 4*ks + lq][i3][j3], as stored
#pragma unroll
      for (int ks = 0; ks < G::KS2; ++ks) {
        const size_t at = a0 + (size_t)16 * ks * sh.n3;
        x.a[ks] = BF16 ? bf16_to_float(g3b[at]) : g3[at];
      }
    };
    auto compute = [&](const Item &x) __attribute__((always_inline)) {
      const float *bp = P12s + x.p * G::PS + lm * G::Rp + lq;
      f32x4 o[G::NT2];
#pragma unroll
      for (int nt = 0; nt < G::NT2; ++nt) o[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < G::KS2; ++ks)
#pragma unroll
        for (int nt = 0; nt < G::NT2; ++nt)
          o[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x.a[ks], bp[16 * nt * G::Rp + 4 * ks], o[nt], 0, 0, 0);
      // C[m = (row = lq, j3 = v)][n = cc]: one float4 of row ubase+lq at columns (j1, j2, 0..3)
      if (lq < x.nrow) {
#pragma unroll
        for (int nt = 0; nt < G::NT2; ++nt) {
          const int cc = 16 * nt + lm, j1 = cc / G::JW, j2 = j2base + (cc - j1 * G::JW);
          *reinterpret_cast<float4 *>(rowbuf + (size_t)(x.ubase + lq) * G::D + (j1 * D2 + j2) * 4) =
              make_float4(o[nt][0], o[nt][1], o[nt][2], o[nt][3]);
        }
      }
    };
    constexpr int NWV = FTHR / 64;
    // (four wavefronts per SIMD cover each other's gathers; keeping a second item's operands in
    // registers to prefetch it was measured and costs more in spilled registers than it hides)
    for (int it = wave; it < total; it += NWV) {
      Item x;
      fetch(it, x);
      compute(x);
    }
    if (more && refill) {  // uniform: the staged plan entries are used up, fetch the next 64
      __syncthreads();  // every reader of the plan entries is done
      fetch_meta(cs + TT_MP);
      __syncthreads();
      fetch_chunk(0);
      stage_chunk(par ^ 1, 0);
    }
    par ^= 1;
  }
}

template <int R1, int R2, int D2, bool P12OUT, bool BF16 = false>
tt_status launch(const TTBatch &b, hipStream_t s) {
  using G = FwdGeom<R1, R2, D2>;
  const size_t lds = G::LDS_FLOATS * sizeof(float);
  // once per process and kernel instantiation; calls may come from several host threads
  static std::once_flag once;
  static bool configured = false;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_fwd_mfma<false, R1, R2, D2, P12OUT, BF16>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                 hipFuncSetAttribute(reinterpret_cast<const void *>(&k_fwd_mfma<true, R1, R2, D2, P12OUT, BF16>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
  });
  if (!configured) return TT_ERR_HIP;
  // Two workgroups fit on each of the 256 compute units.  A table with fewer (i2, strip) pairs than
  // that deals the chunks of each pair to several workgroups (the widest table of a batch decides).
  const long long n2p8 = tt_batch_max(b, [](const TTDev &d) { return (long long)((d.sh.n2 + 7) & ~7); });
  int split = (int)(TT_FWD_WG_TARGET / (n2p8 * G::NSTRIP));
  split = split < 1 ? 1 : (split > TT_FWD_MAX_SPLIT ? TT_FWD_MAX_SPLIT : split);
  const long long blocks = n2p8 * G::NSTRIP * split;
  // timed by the kernel's own begin and end stamps when a profile object asks
  TTProfScope prof(&b.host[0].plan, P12OUT ? TT_KERNEL_P12_FILL : TT_KERNEL_FWD_CONTRACT, s, false);
  if (b.dev)
    hipExtLaunchKernelGGL((k_fwd_mfma<true, R1, R2, D2, P12OUT, BF16>), dim3((unsigned)blocks, (unsigned)b.T),
                          dim3(FTHR), lds, s, prof.start(), prof.stop(), 0, TTArg<true>{b.dev}, split);
  else
    hipExtLaunchKernelGGL((k_fwd_mfma<false, R1, R2, D2, P12OUT, BF16>), dim3((unsigned)blocks), dim3(FTHR), lds, s,
                          prof.start(), prof.stop(), 0, TTArg<false>{b.host[0]}, split);
  return tt_launch_status();
}

}  // namespace

bool ttk_forward_mfma_supported(const TTShape &sh) {
  if (sh.d1 != 4 || sh.d3 != 4 || sh.d2 != 8) return false;
  return (sh.R1 == 32 && sh.R2 == 32) || (sh.R1 == 64 && sh.R2 == 64);
}

tt_status ttk_forward_mfma(const TTBatch &b, hipStream_t s) {
  if (b.host[0].sh.R1 == 32) return launch<32, 32, 8, false>(b, s);
  return launch<64, 64, 8, false>(b, s);
}

tt_status ttk_forward_mfma_bf16(const TTBatch &b, hipStream_t s) {
  if (b.host[0].sh.R1 == 32) return launch<32, 32, 8, false, true>(b, s);
  return launch<64, 64, 8, false, true>(b, s);
}

tt_status ttk_forward_mfma_p12(const TTBatch &b, hipStream_t s) {
  if (b.host[0].sh.R1 == 32) return launch<32, 32, 8, true>(b, s);
  return launch<64, 64, 8, true>(b, s);
}
