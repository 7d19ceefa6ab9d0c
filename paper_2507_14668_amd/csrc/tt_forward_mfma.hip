// MFMA forward contraction for the TT embedding bag (paper Section III-B/III-C), gfx950.
//
// Work is grouped by i2: the distinct prefixes (i1, i2) of the batch that share an i2 are cut into
// chunks of TT_MP = 8, and one workgroup owns one (chunk, 256-column strip of the core-1 slice
// G2[:, i2, :, :]).  For a chunk
//   F1: P12[(p,j1)][(j2,r2)] = sum_r1 G1[i1_p][j1][r1] * G2[r1][i2][j2][r2]
// is a 32 x R1 x 256 GEMM on v_mfma_f32_16x16x4_f32 (A = the 8 core-0 slices staged in LDS,
// B = the strip, loaded straight into registers), so every core-1 element loaded from memory
// feeds all prefixes of the chunk instead of one.  The product is written to LDS and
//   F2: row[(j1,j2)][j3] = sum_r2 P12[(j1,j2)][r2] * G3[r2][i3][j3]
// runs per (prefix, four distinct rows) as a 16 x R2 x (4*JW) MFMA GEMM whose A operand is
// gathered from core 2; rows are stored as float4.
//
// Operand layout of __builtin_amdgcn_mfma_f32_16x16x4f32 (D = A[16x4] * B[4x16] + C):
//   lane l supplies A[m = l%16][k = l/16] and B[k = l/16][n = l%16];
//   lane l holds C[m = 4*(l/16) + v][n = l%16] in component v of its float4.
#include <mutex>

#include "tt_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MT = TT_MP / 4;  // 16-row MFMA tiles of (prefix, j1) rows per chunk

template <int R1, int R2, int D2>
struct FwdGeom {
  static constexpr int JW = 256 / R2;      // j2 values covered by one 256-column strip
  static constexpr int NSTRIP = D2 / JW;   // strips per i2
  static constexpr int S2 = D2 * R2;       // floats per r1-chunk of a core-1 slice
  static constexpr int RS = R1 + 4;        // LDS row stride of the core-0 tile
  static constexpr int Rp = R2 + 4;        // LDS row stride of a P12 row [(j1,j2)][r2]
  static constexpr int CC = 4 * JW;        // (j1, j2) columns per strip
  // LDS stride between the P12 blocks of two prefixes.  F1 stores one value per lane at
  // [prefix = lq (+4 mt)][...][r2 = 4*lm + nt]: 4*lm covers every fourth bank, so the stride is
  // 17 mod 32 (lq -> 0, 17, 2, 19: the four residues mod 4) and a store is 2-way at worst.
  static constexpr int PS = CC * Rp + 17;
  static constexpr int KS1 = R1 / 4, KS2 = R2 / 4;
  static constexpr int NT2 = CC / 16;
  static constexpr int D = 4 * D2 * 4;
  static constexpr size_t LDS_FLOATS = (size_t)TT_MP * PS;
  static_assert(256 % R2 == 0 && D2 % JW == 0 && R1 % 4 == 0 && CC % 16 == 0, "unsupported shape");
  static_assert(TT_MP * 4 * RS <= TT_MP * PS && TT_MP % 4 == 0, "core-0 tile must fit in the P12 area it aliases");
};

constexpr int FWD_I3_STAGE = TT_BLOCK / TT_MP;  // i3 of the first 32 distinct rows of each prefix is staged in LDS

template <bool BATCHED, int R1, int R2, int D2>
__global__ void __launch_bounds__(TT_BLOCK)
k_fwd_mfma(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const float *__restrict__ g1 = d.g[0], *__restrict__ g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int32_t *__restrict__ counts = d.plan.counts, *__restrict__ uniq_row = d.plan.uniq_row;
  const int4 *__restrict__ chunk_rec = reinterpret_cast<const int4 *>(d.plan.chunk_i2);
  const int4 *__restrict__ pref_meta = reinterpret_cast<const int4 *>(d.plan.pref_meta);
  float *__restrict__ rowbuf = d.plan.rowbuf;
  using G = FwdGeom<R1, R2, D2>;
  extern __shared__ float lds[];
  float *As = lds;    // [32][RS]  core-0 slices of the chunk (dead once F1 is done)
  float *P12s = lds;  // [8][PS]   prefix products of the chunk
  __shared__ int s_i1[TT_MP], s_u0[TT_MP], s_nr[TT_MP], s_item_off[TT_MP + 1];
  __shared__ int s_i3[TT_MP][FWD_I3_STAGE];

  const int nchunks = counts[5];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lm = lane & 15, lq = lane >> 4;

  for (int work = blockIdx.x; work < nchunks * G::NSTRIP; work += gridDim.x) {
    const int chunk = work / G::NSTRIP, strip = work - chunk * G::NSTRIP;
    const int j2base = strip * G::JW;
    const int4 rec = chunk_rec[chunk];  // i2, position of the chunk's first prefix, its prefixes
    const int i2 = rec.x, cs = rec.y, cnt = rec.z;

    // This wavefront's 64 columns of the strip of G2[:, i2], all r1 (B operand of F1), as one
    // float4 per row and lane: lane lm holds columns 4*lm .. 4*lm + 3, and MFMA tile nt takes
    // component nt, i.e. tile column lm stands for strip column 64*wave + 4*lm + nt.
    float4 bq[G::KS1];
#pragma unroll
    for (int ks = 0; ks < G::KS1; ++ks)
      bq[ks] = *reinterpret_cast<const float4 *>(g2 + ((size_t)(4 * ks + lq) * sh.n2 + i2) * G::S2 + strip * 256 +
                                                 64 * wave + 4 * lm);

    __syncthreads();  // the previous work item's readers of P12s / s_* are done
    if (threadIdx.x < TT_MP) {
      int i1 = -1, u0 = 0, nr = 0;
      if ((int)threadIdx.x < cnt) {
        const int4 m = pref_meta[cs + threadIdx.x];  // i1, first row slot, rows, prefix slot
        i1 = m.x; u0 = m.y; nr = m.z;
      }
      s_i1[threadIdx.x] = i1;
      s_u0[threadIdx.x] = u0;
      s_nr[threadIdx.x] = nr;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int run = 0;
      for (int p = 0; p < TT_MP; ++p) { s_item_off[p] = run; run += (s_nr[p] + 3) >> 2; }
      s_item_off[TT_MP] = run;
    }
    {  // i3 of the first rows of every prefix (F2 would otherwise start each item with this load)
      const int p = threadIdx.x / FWD_I3_STAGE, r = threadIdx.x - p * FWD_I3_STAGE;
      s_i3[p][r] = uniq_row[s_u0[p] + (r < s_nr[p] ? r : 0)] % sh.n3;
    }
    // stage the core-0 slices: As[(p*4 + j1)][r1], zero rows for the unused tail of the chunk
    for (int e = threadIdx.x; e < TT_MP * 4 * R1; e += TT_BLOCK) {
      const int row = e / R1, r1 = e - row * R1;
      const int i1 = s_i1[row >> 2];
      As[row * G::RS + r1] = i1 >= 0 ? g1[(size_t)i1 * (4 * R1) + (row & 3) * R1 + r1] : 0.f;
    }
    __syncthreads();

    // ---- F1: C[32 x 64 per wave] on MFMA -----------------------------------------------------
    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < G::KS1; ++ks) {
      float av[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) av[mt] = As[(16 * mt + lm) * G::RS + 4 * ks + lq];
      const float bv[4] = {bq[ks].x, bq[ks].y, bq[ks].z, bq[ks].w};
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mt], bv[nt], acc[mt][nt], 0, 0, 0);
    }
    __syncthreads();  // every wave has finished reading As before P12s overwrites it
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int p = 4 * mt + lq;  // C row m = 4*lq + v  ->  prefix 4*mt + lq, j1 = v
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        const int cl = 64 * wave + 4 * lm + nt, j2loc = cl / R2, r2 = cl - j2loc * R2;
#pragma unroll
        for (int v = 0; v < 4; ++v)
          P12s[p * G::PS + (v * G::JW + j2loc) * G::Rp + r2] = acc[mt][nt][v];
      }
    }
    __syncthreads();

    // ---- F2: items = (prefix, four distinct rows), dealt round-robin to the wavefronts -------
    // The core-2 operand of a wavefront's next item is requested before the MFMAs of the current
    // one (unconditionally: past the last item the last one is requested again and not used).
    const int total = s_item_off[TT_MP];
    struct Item { int p, ubase, nrow; float a[G::KS2]; };
    auto fetch = [&](int it, Item &x) __attribute__((always_inline)) {
      it = it < total ? it : total - 1;
      int p = 0;
#pragma unroll
      for (int k = 1; k < TT_MP; ++k) p += (s_item_off[k] <= it) ? 1 : 0;
      // p = number of k in 1..TT_MP-1 with item_off[k] <= it = the prefix whose range holds `it`
      const int quad = it - s_item_off[p];
      x.p = p;
      x.ubase = s_u0[p] + 4 * quad;
      const int left = s_nr[p] - 4 * quad;
      x.nrow = left < 4 ? left : 4;
      // A operand: G3[r2][i3(row)][j3], m = (row, j3) = lm, k = r2
      const int arow = 4 * quad + ((lm >> 2) < x.nrow ? (lm >> 2) : x.nrow - 1);
      const int i3 = arow < FWD_I3_STAGE ? s_i3[p][arow] : uniq_row[s_u0[p] + arow] % sh.n3;
      const float *ap = g3 + ((size_t)lq * sh.n3 + i3) * 4 + (lm & 3);  // G3[r2 = 4*ks + lq][i3][j3], as stored
#pragma unroll
      for (int ks = 0; ks < G::KS2; ++ks) x.a[ks] = ap[(size_t)16 * ks * sh.n3];
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
    constexpr int NWV = TT_BLOCK / 64;
    if (wave < total) {  // uniform per wavefront
      Item xa, xb;
      fetch(wave, xa);
      int it = wave;
      while (true) {  // written out twice so that both operand sets stay in registers
        fetch(it + NWV, xb);
        compute(xa);
        if ((it += NWV) >= total) break;
        fetch(it + NWV, xa);
        compute(xb);
        if ((it += NWV) >= total) break;
      }
    }
  }
}

template <int R1, int R2, int D2>
tt_status launch(const TTBatch &b, hipStream_t s) {
  using G = FwdGeom<R1, R2, D2>;
  const size_t lds = G::LDS_FLOATS * sizeof(float);
  // once per process and kernel instantiation; calls may come from several host threads
  static std::once_flag once;
  static bool configured = false;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_fwd_mfma<false, R1, R2, D2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                 hipFuncSetAttribute(reinterpret_cast<const void *>(&k_fwd_mfma<true, R1, R2, D2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
  });
  if (!configured) return TT_ERR_HIP;
  // upper bound of the chunk count: every i2 adds at most one partly filled chunk
  long long blocks = tt_batch_max(b, [](const TTDev &d) {
    return (long long)(d.plan.max_prefixes / TT_MP + d.sh.n2) * G::NSTRIP; });
  if (blocks > 8192) blocks = 8192;  // grid-stride loop covers the rest
  TTProfScope prof(&b.host[0].plan, TT_KERNEL_FWD_CONTRACT, s);
  if (b.dev)
    hipLaunchKernelGGL((k_fwd_mfma<true, R1, R2, D2>), dim3((unsigned)blocks, (unsigned)b.T),
                       dim3(TT_BLOCK), lds, s, TTArg<true>{b.dev});
  else
    hipLaunchKernelGGL((k_fwd_mfma<false, R1, R2, D2>), dim3((unsigned)blocks), dim3(TT_BLOCK), lds, s,
                       TTArg<false>{b.host[0]});
  return tt_launch_status();
}

}  // namespace

bool ttk_forward_mfma_supported(const TTShape &sh) {
  if (sh.d1 != 4 || sh.d3 != 4 || sh.d2 != 8) return false;
  return (sh.R1 == 32 && sh.R2 == 32) || (sh.R1 == 64 && sh.R2 == 64);
}

tt_status ttk_forward_mfma(const TTBatch &b, hipStream_t s) {
  if (b.host[0].sh.R1 == 32) return launch<32, 32, 8>(b, s);
  return launch<64, 64, 8>(b, s);
}
