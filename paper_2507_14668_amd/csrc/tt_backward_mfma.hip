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
#define TT_I3_STAGE 32  // i3 of the first 32 distinct rows of each prefix is staged in LDS


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
  static constexpr int GS = D + 16;        // gs   [32 rows][D]   merged gradients of a row batch
  static constexpr int G3S = S3 + 16;      // g3s  [32 rows][S3]  their core-2 slices
  static constexpr int OFF_GS = OFF_P12 + TT_MP * PS;
  static constexpr int OFF_G3S = OFF_GS + 32 * GS;
  static constexpr size_t LDS_FLOATS = (size_t)OFF_G3S + 32 * G3S;
  static_assert(256 % R2 == 0 && D2 % JW == 0 && R1 % 16 == 0 && R2 % 16 == 0 && CC % 16 == 0, "shape");
  static_assert(4 * 32 * R1 <= TT_MP * PS, "T1 partials alias the P12 area");
  static_assert(TT_MP == 8, "chunk geometry: two 16-row tiles of (prefix, j1) rows");
};

#define TT_META 64  // prefixes whose plan entries are fetched into LDS in one go (8 chunks)

template <int R1, int R2, int D2>
__global__ void __launch_bounds__(TT_BLOCK)
k_bwd_mfma(TTShape sh, const float *__restrict__ g1, const float *__restrict__ g2,
           const float *__restrict__ g3t, const int32_t *__restrict__ uniq_pref,
           const int32_t *__restrict__ pref_seg, const int32_t *__restrict__ uniq_row,
           const int32_t *__restrict__ prefs_by_i2, const int32_t *__restrict__ i2_seg,
           const float *__restrict__ gagg, float *__restrict__ t3buf, float *__restrict__ t1buf,
           float *__restrict__ dg2, float *__restrict__ dbg) {
  using G = BwdGeom<R1, R2, D2>;
  constexpr int GPT = (32 * R1) / TT_BLOCK;  // core-0 tile elements per thread
  constexpr int T3_SPLIT = 4 / G::NTH;       // wave groups that alternate over the row quads for T3
  static_assert(G::MT2 * G::NTH == 4, "one H tile per wavefront");
  extern __shared__ float lds[];
  float *As = lds, *AsT = lds + G::OFF_AST, *Hs = lds + G::OFF_HS, *P12sT = lds + G::OFF_P12;
  float *T1s = P12sT;  // [4 waves][32][R1], used after the chunk's last reader of P12sT
  float *gsm = lds + G::OFF_GS, *g3sm = lds + G::OFF_G3S;
  __shared__ int s_item_off[TT_MP + 1];
  __shared__ int s_q[TT_META], s_i1[TT_META], s_u0[TT_META], s_nr[TT_META];
  __shared__ int s_i3[TT_MP][TT_I3_STAGE];

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

#ifdef TT_DBG_TIMING
  long long tph[6] = {0, 0, 0, 0, 0, 0}, tlast = clock64();
#define TT_TICK(k) { long long tn = clock64(); tph[k] += tn - tlast; tlast = tn; }
#else
#define TT_TICK(k)
#endif
  f32x4 acc2[G::NT1][4];  // dG2[m = r1][n = c], persistent over the chunks
#pragma unroll
  for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc2[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Global-memory operands of the NEXT chunk (core-0 rows, i3 of its first rows) are fetched into
  // registers while the current chunk computes, so staging a chunk costs LDS writes only.
  float g1n[GPT];
  int i3n = 0;
  auto fetch_meta = [&](int base) __attribute__((always_inline)) {  // plan entries of prefixes base .. base+63 -> LDS
    if (threadIdx.x < TT_META) {
      int q = -1, i1 = -1, u0 = 0, nr = 0;
      if (base + (int)threadIdx.x < seg1) {
        q = prefs_by_i2[base + threadIdx.x];
        i1 = uniq_pref[q] / sh.n2;
        u0 = pref_seg[q];
        nr = pref_seg[q + 1] - u0;
      }
      s_q[threadIdx.x] = q; s_i1[threadIdx.x] = i1; s_u0[threadIdx.x] = u0; s_nr[threadIdx.x] = nr;
    }
  };
  auto fetch_chunk = [&](int mo) __attribute__((always_inline)) {  // mo = offset of the chunk inside the staged plan entries
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int e = threadIdx.x + k * TT_BLOCK, row = e / R1, r1 = e - row * R1;
      const int i1 = s_i1[mo + (row >> 2)];
      g1n[k] = i1 >= 0 ? g1[(size_t)i1 * G::S1 + (row & 3) * R1 + r1] : 0.f;
    }
    const int p = threadIdx.x / TT_I3_STAGE, r = threadIdx.x - p * TT_I3_STAGE;
    i3n = r < s_nr[mo + p] ? uniq_row[s_u0[mo + p] + r] % sh.n3 : 0;
  };
  static_assert(TT_MP * TT_I3_STAGE == TT_BLOCK, "one staged i3 per thread");

  fetch_meta(seg0);
  __syncthreads();
  fetch_chunk(0);

  for (int cs = seg0; cs < seg1; cs += TT_MP) {
    const int cnt = (seg1 - cs) < TT_MP ? (seg1 - cs) : TT_MP;
    const int mo = (cs - seg0) % TT_META;  // this chunk's offset in s_q / s_i1 / s_u0 / s_nr
    __syncthreads();  // previous chunk: T1 partials read, Hs / AsT / s_i3 consumed
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int e = threadIdx.x + k * TT_BLOCK, row = e / R1, r1 = e - row * R1;
      As[row * G::RS + r1] = g1n[k];
      AsT[r1 * G::RT + row] = g1n[k];
    }
    s_i3[threadIdx.x / TT_I3_STAGE][threadIdx.x % TT_I3_STAGE] = i3n;
    if (threadIdx.x == 0) {  // quads per prefix of this chunk, running total
      int run = 0;
      for (int p = 0; p < TT_MP; ++p) {
        s_item_off[p] = run;
        if (p < cnt) run += (s_nr[mo + p] + 3) >> 2;
      }
      s_item_off[TT_MP] = run;
    }
    for (int e = threadIdx.x; e < 32 * 256; e += TT_BLOCK)  // unused prefixes contribute zeros
      if ((e >> 10) >= cnt) Hs[(e >> 8) * G::HS + (e & 255)] = 0.f;
    __syncthreads();
    TT_TICK(0)

    // Row batches: the merged gradients and core-2 slices of up to 32 distinct rows (8 quads) are
    // brought into LDS by all 256 threads at once (one memory latency per batch instead of one
    // per quad).  The loads of the chunk's first batch are issued before F1 and land in LDS after
    // it, so F1's MFMAs hide their latency.
    const int total_items = s_item_off[TT_MP];
    float4 rg[4], r3[G::S3 / 32];
#pragma unroll
    for (int k = 0; k < 4; ++k) rg[k] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < G::S3 / 32; ++k) r3[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    int rvalid = 0;
    auto issue_batch = [&](int b) __attribute__((always_inline)) {  // global -> registers; thread t serves row slot t/8
      const int rr = threadIdx.x >> 3, sub = threadIdx.x & 7;
      const int it = 8 * b + (rr >> 2), r = rr & 3;
      rvalid = 0;
      if (it < total_items) {
        int p = 0;
#pragma unroll
        for (int k = 1; k < TT_MP; ++k) p += (s_item_off[k] <= it) ? 1 : 0;
        const int r0 = 4 * (it - s_item_off[p]) + r;
        if (r0 < s_nr[mo + p]) {
          const int u = s_u0[mo + p] + r0;
          const int i3 = r0 < TT_I3_STAGE ? s_i3[p][r0] : uniq_row[u] % sh.n3;
          const float4 *gp = reinterpret_cast<const float4 *>(gagg + (size_t)u * G::D) + sub;
          const float4 *g3p = reinterpret_cast<const float4 *>(g3t + (size_t)i3 * G::S3) + sub;
#pragma unroll
          for (int k = 0; k < 4; ++k) rg[k] = gp[8 * k];
#pragma unroll
          for (int k = 0; k < G::S3 / 32; ++k) r3[k] = g3p[8 * k];
          rvalid = 1;
        }
      }
    };
    auto land_batch = [&]() __attribute__((always_inline)) {  // registers -> LDS
      if (rvalid) {
        const int rr = threadIdx.x >> 3, sub = threadIdx.x & 7;
        float4 *gd = reinterpret_cast<float4 *>(gsm + rr * G::GS) + sub;
        float4 *g3d = reinterpret_cast<float4 *>(g3sm + rr * G::G3S) + sub;
#pragma unroll
        for (int k = 0; k < 4; ++k) gd[8 * k] = rg[k];
#pragma unroll
        for (int k = 0; k < G::S3 / 32; ++k) g3d[8 * k] = r3[k];
      }
    };
    issue_batch(0);

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
    land_batch();
    // next chunk's operands: requested now, consumed at the top of the next iteration
    if (cs + TT_MP < seg1 && mo + TT_MP != TT_META) fetch_chunk(mo + TT_MP);
    __syncthreads();
    TT_TICK(1)

    // ---- T3 and H over the distinct rows of the chunk, one quad (<= 4 rows of a prefix) at a time
    // Every wavefront walks the same quads but owns one 16x16 tile of the outputs: tile (hmt, hnt)
    // of H for every row, and tile hnt of T3 for every T3_SPLIT-th quad.  The split is by output
    // tile, not by prefix, so a prefix with hundreds of rows is shared by all four wavefronts and
    // no partial sums have to be combined.
    {
      const int hmt = wave / G::NTH, hnt = wave % G::NTH;
      const int hcol = ((16 * hmt + lm) / G::JW) * D2 + j2base + ((16 * hmt + lm) % G::JW);
      f32x4 hacc = (f32x4){0.f, 0.f, 0.f, 0.f};
      const int nbatch = (total_items + 7) >> 3;
      for (int b = 0; b < nbatch; ++b) {
        if (b > 0) {  // uniform: further batches of a row-rich chunk (latency exposed)
          __syncthreads();
          issue_batch(b);
          land_batch();
          __syncthreads();
        }
        const int it_end = (8 * b + 8) < total_items ? (8 * b + 8) : total_items;
        for (int it = 8 * b; it < it_end; ++it) {
          int p = 0;
#pragma unroll
          for (int k = 1; k < TT_MP; ++k) p += (s_item_off[k] <= it) ? 1 : 0;
          const int quad = it - s_item_off[p];
          const int nr = s_nr[mo + p], ubase = s_u0[mo + p] + 4 * quad;
          const int nrow = (nr - 4 * quad) < 4 ? (nr - 4 * quad) : 4;
          const float *gq = gsm + ((it & 7) * 4) * G::GS;     // the quad's four gradient rows
          const float *g3q = g3sm + ((it & 7) * 4) * G::G3S;  // and core-2 slices
          if ((it % T3_SPLIT) == hmt) {  // T3: M = (row, j3) = lm, N = r2 tile hnt, K = cc
            const float *ga = gq + (lm >> 2) * G::GS + (lm & 3);
            const float *pb = P12sT + p * G::PS + (16 * hnt + lm) * G::CP + lq;
            f32x4 t3 = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < G::KS3; ++ks) {
              const int cc = 4 * ks + lq, col = (cc / G::JW) * D2 + j2base + (cc % G::JW);
              t3 = MFMA(ga[col * 4], pb[4 * ks], t3);
            }
            if (lq < nrow)
              *reinterpret_cast<float4 *>(t3buf + ((size_t)(ubase + lq) * G::NSTRIP + strip) * G::S3 +
                                          (16 * hnt + lm) * 4) = make_float4(t3[0], t3[1], t3[2], t3[3]);
          }
          // H tile (hmt, hnt): M = cc, N = r2, K = j3 (one distinct row per MFMA step)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (r < nrow)
              hacc = MFMA(gq[r * G::GS + hcol * 4 + lq], g3q[r * G::G3S + (16 * hnt + lm) * 4 + lq], hacc);
          if (4 * quad + 4 >= nr) {  // last quad of the prefix: H[cc = 16*hmt + 4*lq + v][r2]
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int c2 = 16 * hmt + 4 * lq + v, j1 = c2 / G::JW, j2loc = c2 - j1 * G::JW;
              Hs[(p * 4 + j1) * G::HS + j2loc * R2 + 16 * hnt + lm] = hacc[v];
            }
            hacc = (f32x4){0.f, 0.f, 0.f, 0.f};
          }
        }
      }
    }
    TT_TICK(2)
    __syncthreads();
    TT_TICK(3)

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
    TT_TICK(4)
    // fold the four K-partials of T1 in wave order and store one contribution per prefix
    for (int e = threadIdx.x; e < 32 * R1; e += TT_BLOCK) {
      const int row = e / R1, p = row >> 2;
      if (p < cnt) {
        const float sum = ((T1s[e] + T1s[32 * R1 + e]) + T1s[2 * 32 * R1 + e]) + T1s[3 * 32 * R1 + e];
        t1buf[((size_t)s_q[mo + p] * G::NSTRIP + strip) * G::S1 + (row & 3) * R1 + (e - row * R1)] = sum;
      }
    }
    if (cs + TT_MP < seg1 && mo + TT_MP == TT_META) {  // uniform: refill the staged plan entries
      __syncthreads();
      fetch_meta(cs + TT_MP);
      __syncthreads();
      fetch_chunk(0);
    }
  }

#ifdef TT_DBG_TIMING
  if (lane == 0) {
    TT_TICK(5)
    for (int k = 0; k < 6; ++k) dbg[(blockIdx.x * 4 + wave) * 8 + k] = (float)tph[k];
    dbg[(blockIdx.x * 4 + wave) * 8 + 6] = (float)(seg1 - seg0);
  }
#endif
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
                     t->core[0], t->core[1], plan->g3t, plan->uniq_pref, plan->pref_seg,
                     plan->uniq_row, plan->prefs_by_i2, plan->i2_seg, plan->gagg, plan->t3buf,
                     plan->t1buf, dg2, plan->hbuf);
  return tt_launch_status();
}

}  // namespace

int ttk_mfma_strips(const TTShape &sh) {
  return ttk_forward_mfma_supported(sh) ? (sh.d2 * sh.R2) / 256 : 1;
}

tt_status ttk_backward_mfma(const TTShape &sh, const tt_table *t, const tt_plan *plan, float *dg2,
                            hipStream_t s) {
  tt_status st = ttk_pack_g3(sh, t, plan, s);
  if (st != TT_OK) return st;
  if (sh.R1 == 32) return launch<32, 32, 8>(sh, t, plan, dg2, s);
  return launch<64, 64, 8>(sh, t, plan, dg2, s);
}
