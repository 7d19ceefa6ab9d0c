// MFMA backward contractions for the TT embedding bag (paper Section III-D backward equation,
// after the in-advance gradient aggregation of Section III-E), gfx950.
//
// One workgroup owns one (i2, 256-column strip of the core-1 slice G2[:, i2, :, :]) and walks the
// distinct prefixes (i1, i2) of the batch in chunks of TT_MP = 8.  With g = the merged output
// gradient of a distinct row and c = (j2, r2) a column of the strip, per chunk it forms
//   F1  P12[(p,j1)][c]  = sum_r1 G1[i1_p][j1][r1] G2[r1][i2][c]            (recomputed, LDS)
//   T3  t3[u][r2][j3]   = sum_{j1,j2 in strip} P12[p][j1][j2][r2] g[u][j1][j2][j3]   (per row)
//   H   H[p][j1][c]     = sum_{rows u of p} sum_j3 g[u][j1][j2][j3] G3[r2][i3_u][j3]
//   T1  t1[p][j1][r1]   = sum_{c in strip} H[p][j1][c] G2[r1][i2][c]                  (per prefix)
//   dG2[r1][i2][c]     += sum_{p in chunk} sum_j1 G1[i1_p][j1][r1] H[p][j1][c]
// all on v_mfma_f32_16x16x4_f32.  dG2 stays in accumulator registers over all chunks of the i2
// and is written once (no atomics, no partial buffers); t3 / t1 are per-row / per-prefix
// contributions (one per strip) that sorted segmented sums fold into dG3 / dG1 afterwards.
// Both views of the G2 strip (B operand of F1: lanes along c; B operand of T1: lanes along r1)
// are loaded into registers once per workgroup.
//
// MFMA operand layout (D = A[16x4] * B[4x16] + C): lane l supplies A[m = l%16][k = l/16] and
// B[k = l/16][n = l%16] and holds C[m = 4*(l/16) + v][n = l%16] in component v.
#include "tt_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)
#define TT_I3_STAGE 16  // i3 of the first 16 distinct rows of each prefix is staged in LDS

template <int R1, int R2, int D2>
struct BwdGeom {
  static constexpr int JW = 256 / R2;      // j2 values covered by one 256-column strip
  static constexpr int NSTRIP = D2 / JW;
  static constexpr int S2 = D2 * R2;
  static constexpr int CC = 4 * JW;        // (j1, j2) columns per strip
  static constexpr int RS = R1 + 4;        // As   [32 (p,j1)][R1]    lanes along rows, k along r1
  static constexpr int RT = 36;            // AsT  [R1][32 (p,j1)]    lanes along r1, k along rows
  static constexpr int CP = CC + 4;        // P12sT row [r2][cc]      lanes along r2, k along cc
  static constexpr int PS = R2 * CP + 1;   // stride between the P12sT blocks of two prefixes
  static constexpr int HS = 260;           // Hs   [32 (p,j1)][256 c]
  static constexpr int KS1 = R1 / 4, NT1 = R1 / 16, NTH = R2 / 16, MT2 = CC / 16, KS3 = CC / 4;
  static constexpr int D = 4 * D2 * 4, S3 = R2 * 4, S1 = 4 * R1;
  static constexpr int OFF_AST = 32 * RS;
  static constexpr int OFF_HS = OFF_AST + R1 * RT;
  static constexpr int OFF_P12 = OFF_HS + 32 * HS;
  static constexpr size_t LDS_FLOATS = (size_t)OFF_P12 + TT_MP * PS;
  static_assert(256 % R2 == 0 && D2 % JW == 0 && R1 % 16 == 0 && R2 % 16 == 0 && CC % 16 == 0, "shape");
  static_assert(4 * 32 * R1 <= TT_MP * PS, "T1 partials alias the P12 area");
  static_assert(TT_MP == 8, "chunk geometry: two 16-row tiles of (prefix, j1) rows");
};

template <int R1, int R2, int D2>
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_mfma(TTShape sh, const float *__restrict__ g1, const float *__restrict__ g2,
           const float *__restrict__ g3, const int32_t *__restrict__ uniq_pref,
           const int32_t *__restrict__ pref_seg, const int32_t *__restrict__ uniq_row,
           const int32_t *__restrict__ prefs_by_i2, const int32_t *__restrict__ i2_seg,
           const float *__restrict__ gagg, float *__restrict__ t3buf, float *__restrict__ t1buf,
           float *__restrict__ dg2) {
  using G = BwdGeom<R1, R2, D2>;
  extern __shared__ float lds[];
  float *As = lds, *AsT = lds + G::OFF_AST, *Hs = lds + G::OFF_HS, *P12sT = lds + G::OFF_P12;
  float *T1s = P12sT;  // [4 waves][32][R1], used after the chunk's last reader of P12sT
  __shared__ int s_q[TT_MP], s_i1[TT_MP], s_u0[TT_MP], s_nr[TT_MP], s_i3[TT_MP][TT_I3_STAGE];

  const int i2 = blockIdx.x / G::NSTRIP, strip = blockIdx.x - i2 * G::NSTRIP;
  const int j2base = strip * G::JW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lm = lane & 15, lq = lane >> 4;
  const int seg0 = i2_seg[i2], seg1 = i2_seg[i2 + 1];
  const size_t strip_col = (size_t)i2 * G::S2 + strip * 256;  // + r1*n2*S2 + c

  if (seg0 == seg1) {  // uniform: no lookup touches this i2, its gradient strip is zero
    for (int e = threadIdx.x; e < R1 * 256; e += TT_BLOCK)
      dg2[(size_t)(e >> 8) * sh.n2 * G::S2 + strip_col + (e & 255)] = 0.f;
    return;
  }

  // both register views of this wave's 64 columns of the strip
  float breg[G::KS1][4];       // F1: B[k = r1][n = c]
  float breg2[16][G::NT1];     // T1: B[k = c][n = r1]
#pragma unroll
  for (int ks = 0; ks < G::KS1; ++ks)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
      breg[ks][nt] = g2[(size_t)(4 * ks + lq) * sh.n2 * G::S2 + strip_col + 64 * wave + 16 * nt + lm];
#pragma unroll
  for (int ks = 0; ks < 16; ++ks)
#pragma unroll
    for (int nt = 0; nt < G::NT1; ++nt)
      breg2[ks][nt] = g2[(size_t)(16 * nt + lm) * sh.n2 * G::S2 + strip_col + 64 * wave + 4 * ks + lq];

  f32x4 acc2[G::NT1][4];  // dG2[m = r1][n = c], persistent over the chunks
#pragma unroll
  for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc2[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  for (int cs = seg0; cs < seg1; cs += TT_MP) {
    const int cnt = (seg1 - cs) < TT_MP ? (seg1 - cs) : TT_MP;
    __syncthreads();  // previous chunk: T1 partials read, Hs / AsT consumed
    if (threadIdx.x < TT_MP) {
      int q = -1, i1 = -1, u0 = 0, nr = 0;
      if ((int)threadIdx.x < cnt) {
        q = prefs_by_i2[cs + threadIdx.x];
        i1 = uniq_pref[q] / sh.n2;
        u0 = pref_seg[q];
        nr = pref_seg[q + 1] - u0;
      }
      s_q[threadIdx.x] = q; s_i1[threadIdx.x] = i1; s_u0[threadIdx.x] = u0; s_nr[threadIdx.x] = nr;
    }
    __syncthreads();
    if (threadIdx.x < TT_MP * TT_I3_STAGE) {
      const int p = threadIdx.x / TT_I3_STAGE, r = threadIdx.x - p * TT_I3_STAGE;
      if (r < s_nr[p]) s_i3[p][r] = uniq_row[s_u0[p] + r] % sh.n3;
    }
    for (int e = threadIdx.x; e < 32 * R1; e += TT_BLOCK) {
      const int row = e / R1, r1 = e - row * R1;
      const int i1 = s_i1[row >> 2];
      const float v = i1 >= 0 ? g1[(size_t)i1 * G::S1 + (row & 3) * R1 + r1] : 0.f;
      As[row * G::RS + r1] = v;
      AsT[r1 * G::RT + row] = v;
    }
    for (int e = threadIdx.x; e < 32 * 256; e += TT_BLOCK)  // unused prefixes contribute zeros
      if ((e >> 10) >= cnt) Hs[(e >> 8) * G::HS + (e & 255)] = 0.f;
    __syncthreads();

    // ---- F1: P12 of the chunk -> P12sT[p][r2][cc] ---------------------------------------------
    {
      f32x4 acc[2][4];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < G::KS1; ++ks) {
        float a[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = As[(16 * mt + lm) * G::RS + 4 * ks + lq];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = MFMA(a[mt], breg[ks][nt], acc[mt][nt]);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int p = 4 * mt + lq;  // C row 4*lq + v -> prefix 4*mt + lq, j1 = v
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          const int cl = 64 * wave + 16 * nt + lm, j2loc = cl / R2, r2 = cl - j2loc * R2;
#pragma unroll
          for (int v = 0; v < 4; ++v)
            P12sT[p * G::PS + r2 * G::CP + v * G::JW + j2loc] = acc[mt][nt][v];
        }
      }
    }
    __syncthreads();

    // ---- T3 and H: one wavefront per prefix, its distinct rows four at a time -----------------
    for (int p = wave; p < cnt; p += TT_BLOCK / 64) {
      f32x4 hacc[G::MT2][G::NTH];
#pragma unroll
      for (int mt = 0; mt < G::MT2; ++mt)
#pragma unroll
        for (int nt = 0; nt < G::NTH; ++nt) hacc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const int u0 = s_u0[p], nr = s_nr[p];
      const float *pb = P12sT + p * G::PS + lm * G::CP + lq;
      for (int r0 = 0; r0 < nr; r0 += 4) {
        const int ubase = u0 + r0, nrow = (nr - r0) < 4 ? (nr - r0) : 4;
        // T3: M = (row, j3) = lm, N = r2, K = cc
        {
          const int arow = (lm >> 2) < nrow ? (lm >> 2) : nrow - 1;
          const float *ga = gagg + (size_t)(ubase + arow) * G::D + (lm & 3);
          f32x4 t3[G::NTH];
#pragma unroll
          for (int nt = 0; nt < G::NTH; ++nt) t3[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < G::KS3; ++ks) {
            const int cc = 4 * ks + lq, col = (cc / G::JW) * D2 + j2base + (cc % G::JW);
            const float a = ga[col * 4];
#pragma unroll
            for (int nt = 0; nt < G::NTH; ++nt) t3[nt] = MFMA(a, pb[16 * nt * G::CP + 4 * ks], t3[nt]);
          }
          if (lq < nrow) {
            float *dst = t3buf + ((size_t)(ubase + lq) * G::NSTRIP + strip) * G::S3 + lm * 4;
#pragma unroll
            for (int nt = 0; nt < G::NTH; ++nt)
              *reinterpret_cast<float4 *>(dst + 64 * nt) =
                  make_float4(t3[nt][0], t3[nt][1], t3[nt][2], t3[nt][3]);
          }
        }
        // H: M = cc, N = r2, K = j3 (one row per MFMA step)
        for (int r = 0; r < nrow; ++r) {
          const int u = ubase + r;
          const int i3 = (r0 + r) < TT_I3_STAGE ? s_i3[p][r0 + r] : uniq_row[u] % sh.n3;
          float ah[G::MT2], bh[G::NTH];
#pragma unroll
          for (int mt = 0; mt < G::MT2; ++mt) {
            const int cc = 16 * mt + lm, col = (cc / G::JW) * D2 + j2base + (cc % G::JW);
            ah[mt] = gagg[(size_t)u * G::D + col * 4 + lq];
          }
#pragma unroll
          for (int nt = 0; nt < G::NTH; ++nt)
            bh[nt] = g3[((size_t)(16 * nt + lm) * sh.n3 + i3) * 4 + lq];
#pragma unroll
          for (int mt = 0; mt < G::MT2; ++mt)
#pragma unroll
            for (int nt = 0; nt < G::NTH; ++nt) hacc[mt][nt] = MFMA(ah[mt], bh[nt], hacc[mt][nt]);
        }
      }
      // H[cc = 16*mt + 4*lq + v][r2 = 16*nt + lm] -> Hs[(p, j1)][j2loc*R2 + r2]
#pragma unroll
      for (int mt = 0; mt < G::MT2; ++mt)
#pragma unroll
        for (int nt = 0; nt < G::NTH; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int cc = 16 * mt + 4 * lq + v, j1 = cc / G::JW, j2loc = cc - j1 * G::JW;
            Hs[(p * 4 + j1) * G::HS + j2loc * R2 + 16 * nt + lm] = hacc[mt][nt][v];
          }
    }
    __syncthreads();

    // ---- T1 (K = this wave's 64 columns) and dG2 (N = this wave's 64 columns) -----------------
    {
      f32x4 acc1[2][G::NT1];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < G::NT1; ++nt) acc1[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        float a[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = Hs[(16 * mt + lm) * G::HS + 64 * wave + 4 * ks + lq];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < G::NT1; ++nt) acc1[mt][nt] = MFMA(a[mt], breg2[ks][nt], acc1[mt][nt]);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < G::NT1; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            T1s[(wave * 32 + 16 * mt + 4 * lq + v) * R1 + 16 * nt + lm] = acc1[mt][nt][v];
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      float a[G::NT1], b[4];
#pragma unroll
      for (int mt = 0; mt < G::NT1; ++mt) a[mt] = AsT[(16 * mt + lm) * G::RT + 4 * ks + lq];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) b[nt] = Hs[(4 * ks + lq) * G::HS + 64 * wave + 16 * nt + lm];
#pragma unroll
      for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc2[mt][nt] = MFMA(a[mt], b[nt], acc2[mt][nt]);
    }
    __syncthreads();
    // fold the four K-partials of T1 in wave order and store one contribution per prefix
    for (int e = threadIdx.x; e < 32 * R1; e += TT_BLOCK) {
      const int row = e / R1, p = row >> 2;
      if (p < cnt) {
        const float sum = ((T1s[e] + T1s[32 * R1 + e]) + T1s[2 * 32 * R1 + e]) + T1s[3 * 32 * R1 + e];
        t1buf[((size_t)s_q[p] * G::NSTRIP + strip) * G::S1 + (row & 3) * R1 + (e - row * R1)] = sum;
      }
    }
  }

  // dG2[r1 = 16*mt + 4*lq + v][i2][c = 64*wave + 16*nt + lm], complete for this i2 and strip
#pragma unroll
  for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        dg2[(size_t)(16 * mt + 4 * lq + v) * sh.n2 * G::S2 + strip_col + 64 * wave + 16 * nt + lm] =
            acc2[mt][nt][v];
}

template <int R1, int R2, int D2>
tt_status launch(const TTShape &sh, const tt_table *t, const tt_plan *plan, float *dg2,
                 hipStream_t s) {
  using G = BwdGeom<R1, R2, D2>;
  const size_t lds = G::LDS_FLOATS * sizeof(float);
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bwd_mfma<R1, R2, D2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return TT_ERR_HIP;
    configured = true;
  }
  TTProfScope prof(plan, TT_KERNEL_BWD_CONTRACT, s);
  hipLaunchKernelGGL((k_bwd_mfma<R1, R2, D2>), dim3(sh.n2 * G::NSTRIP), dim3(TT_BLOCK), lds, s, sh,
                     t->core[0], t->core[1], t->core[2], plan->uniq_pref, plan->pref_seg,
                     plan->uniq_row, plan->prefs_by_i2, plan->i2_seg, plan->gagg, plan->t3buf,
                     plan->t1buf, dg2);
  return tt_launch_status();
}

}  // namespace

int ttk_mfma_strips(const TTShape &sh) {
  return ttk_forward_mfma_supported(sh) ? (sh.d2 * sh.R2) / 256 : 1;
}

tt_status ttk_backward_mfma(const TTShape &sh, const tt_table *t, const tt_plan *plan, float *dg2,
                            hipStream_t s) {
  if (sh.R1 == 32) return launch<32, 32, 8>(sh, t, plan, dg2, s);
  return launch<64, 64, 8>(sh, t, plan, dg2, s);
}
