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
// and is written once (no atomics); t3 / t1 are per-row / per-prefix contributions (one per strip)
// that sorted segmented sums fold into dG3 / dG1 afterwards.  Both views of the G2 strip (B operand
// of F1: lanes along c; B operand of T1: lanes along r1) are loaded into registers once per
// workgroup.
//
// A workgroup has eight wavefronts (512 threads), two per SIMD: LDS (155 KB) allows one workgroup
// per compute unit, and with one wavefront per SIMD every instruction that is not an MFMA -- operand
// staging, address arithmetic, stores -- would be issued while the matrix core idles.
//   F1 / dG2   wavefront w owns columns [32w, 32w + 32) of the strip (two 16-column tiles);
//   T1         the four wavefront pairs split K (64 columns each), the two wavefronts of a pair
//              split the r1 tiles; the four K-partials are folded through LDS in pair order;
//   row phase  wavefronts 0-3 accumulate the four H tiles, wavefronts 4-7 form the T3 tiles, so the
//              two wavefronts that share a SIMD issue side by side and no sum crosses wavefronts.
//
// MFMA operand layout (D = A[16x4] * B[4x16] + C): lane l supplies A[m = l%16][k = l/16] and
// B[k = l/16][n = l%16] and holds C[m = 4*(l/16) + v][n = l%16] in component v.
#include <mutex>

#include "tt_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)
constexpr int NTHR = 512;          // threads per workgroup
constexpr int I3_STAGE = NTHR / TT_MP;  // i3 of the first 64 distinct rows of each prefix is staged in LDS
constexpr int META = 64;           // prefixes whose plan entries are fetched into LDS in one go (8 chunks)

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
  static constexpr int NT1H = NT1 / 2;     // r1 tiles of T1 per wavefront of a pair
  static constexpr int D = 4 * D2 * 4, S3 = R2 * 4, S1 = 4 * R1;
  static constexpr int A_FLOATS = 32 * RS + R1 * RT;  // one As + AsT pair
  static constexpr int OFF_AST = 32 * RS;             // AsT inside a pair
  static constexpr int OFF_HS = 2 * A_FLOATS;         // two pairs: current chunk / next chunk
  static constexpr int OFF_P12 = OFF_HS + 32 * HS;
  static constexpr int GS = CC * 4 + 16;   // gs   [32 rows][CC*4] merged gradients of a row batch, strip columns
  static constexpr int G3S = S3 + 16;      // g3s  [32 rows][S3]  their core-2 slices
  static constexpr int OFF_GS = OFF_P12 + TT_MP * PS;
  static constexpr int OFF_G3S = OFF_GS + 32 * GS;
  static constexpr size_t LDS_FLOATS = (size_t)OFF_G3S + 32 * G3S;
  static constexpr int SW = 36;            // row stride of the strip staging tile [R1][32 columns] of a wavefront
  static_assert(256 % R2 == 0 && D2 % JW == 0 && R1 % 32 == 0 && R2 % 16 == 0 && CC % 16 == 0, "shape");
  static_assert(8 * R1 * SW <= 32 * HS + TT_MP * PS, "the strip staging tiles alias the H and P12 areas");
  static_assert(4 * 32 * R1 <= TT_MP * PS, "T1 partials alias the P12 area");
  static_assert(TT_MP == 8 && MT2 * NTH == 4, "chunk geometry: four H tiles, one per wavefront 0-3");
};

template <bool BATCHED, int R1, int R2, int D2>
__global__ void __launch_bounds__(NTHR)
k_bwd_mfma(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  // with the fused update the strip of core 1 this workgroup reads is also the one it rewrites at
  // the end (no other workgroup touches it), so g2 / dg2 may alias and carry no __restrict__
  const float *__restrict__ g1 = d.g[0], *g2 = d.g[1], *__restrict__ g3 = d.g[2];
  const int32_t *__restrict__ uniq_row = d.plan.uniq_row, *__restrict__ i2_seg = d.plan.i2_seg;
  const int4 *__restrict__ pref_meta = reinterpret_cast<const int4 *>(d.plan.pref_meta);
  const float *__restrict__ gagg = d.plan.gagg;
  float *__restrict__ t3buf = d.plan.t3buf, *__restrict__ t1buf = d.plan.t1buf;
  const int fused = d.fused;
  const float lr = d.lr;
  float *dg2 = fused ? const_cast<float *>(d.g[1]) : d.dg[1];
  using G = BwdGeom<R1, R2, D2>;
  constexpr int GPT = (32 * R1) / NTHR;      // core-0 tile elements per thread
  constexpr int T3_SPLIT = 4 / G::NTH;       // T3 wavefront classes that alternate over the row quads
  extern __shared__ float lds[];
  float *Hs = lds + G::OFF_HS, *P12sT = lds + G::OFF_P12;  // As / AsT: two pairs at lds + par*A_FLOATS
  float *T1s = P12sT;  // [4 pairs][32][R1], used after the chunk's last reader of P12sT
  float *gsm = lds + G::OFF_GS, *g3sm = lds + G::OFF_G3S;
  __shared__ int s_item_off[2][TT_MP + 1];
  __shared__ __align__(16) int s_bitem[8][4];  // items of the current row batch: prefix, first row slot, rows, last
  __shared__ int s_q[META], s_i1[META], s_u0[META], s_nr[META];
  __shared__ int s_i3[2][TT_MP][I3_STAGE];

  // workgroup = (i2, strip, part): with split > 1 the chunks of one (i2, strip) are dealt in
  // contiguous runs to `split` workgroups, each of which leaves a partial core-1 gradient
  const int split = d.bwd_split;
  if ((int)blockIdx.x >= sh.n2 * G::NSTRIP * split) return;  // a table of the batch with fewer i2 values
  const int part = blockIdx.x % split, wg = blockIdx.x / split;
  const int i2 = wg / G::NSTRIP, strip = wg - i2 * G::NSTRIP;
  const int j2base = strip * G::JW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lm = lane & 15, lq = lane >> 4;
  const int pair = wave >> 1, half = wave & 1;
  const size_t strip_col = (size_t)i2 * G::S2 + strip * 256;  // + r1*n2*S2 + c
  // The strip is read from memory once, as whole 128-byte rows per wavefront (float4 per lane:
  // eight rows per load).  The loads depend on the workgroup index only and are requested before
  // the plan is looked at, so that their latency overlaps the chain of dependent plan loads.
  f32x4 sreg[R1 / 8];
  {
    const int rsub = lane >> 3, c4 = lane & 7;
#pragma unroll
    for (int i = 0; i < R1 / 8; ++i)
      sreg[i] = *reinterpret_cast<const f32x4 *>(g2 + (size_t)(8 * i + rsub) * sh.n2 * G::S2 + strip_col + 32 * wave + 4 * c4);
  }
  int seg0 = i2_seg[i2], seg1 = i2_seg[i2 + 1];
  const bool touched = seg0 != seg1;
  if (split > 1) {
    const int nch = (seg1 - seg0 + TT_MP - 1) / TT_MP, per = (nch + split - 1) / split;
    const int c0 = part * per, c1 = (c0 + per) < nch ? (c0 + per) : nch;
    const int lo = seg0 + c0 * TT_MP, hi = seg0 + c1 * TT_MP;
    seg1 = c0 < c1 ? (hi < seg1 ? hi : seg1) : seg0;
    seg0 = c0 < c1 ? lo : seg0;
    dg2 = d.plan.dg2part + (size_t)part * R1 * sh.n2 * G::S2;  // partial gradients have the shape of core 1
  }

  if (seg0 == seg1) {  // uniform: no prefix for this workgroup, its gradient strip is zero
    if ((fused && split == 1) || (split > 1 && !touched)) return;  // nothing will read it
    for (int e = threadIdx.x; e < R1 * 256; e += NTHR)
      dg2[(size_t)(e >> 8) * sh.n2 * G::S2 + strip_col + (e & 255)] = 0.f;
    return;
  }

  f32x4 acc2[G::NT1][2];  // dG2[m = r1][n = c], this wavefront's 32 columns, persistent over the chunks
#pragma unroll
  for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) acc2[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Global-memory operands of the NEXT chunk (core-0 rows, i3 of its first rows) are fetched into
  // registers while the current chunk computes, so staging a chunk costs LDS writes only.
  float g1n[GPT];
  int i3n = 0;
  auto fetch_meta = [&](int base) __attribute__((always_inline)) {  // plan entries of prefixes base .. base+63 -> LDS
    if (threadIdx.x < META) {
      int q = -1, i1 = -1, u0 = 0, nr = 0;
      if (base + (int)threadIdx.x < seg1) {
        const int4 m = pref_meta[base + threadIdx.x];  // i1, first row slot, rows, prefix slot
        i1 = m.x; u0 = m.y; nr = m.z; q = m.w;
      }
      s_q[threadIdx.x] = q; s_i1[threadIdx.x] = i1; s_u0[threadIdx.x] = u0; s_nr[threadIdx.x] = nr;
    }
  };
  auto fetch_chunk = [&](int mo) __attribute__((always_inline)) {  // mo = offset of the chunk inside the staged plan entries
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int e = threadIdx.x + k * NTHR, row = e / R1, r1 = e - row * R1;
      // unconditional loads (slice 0 stands in for a prefix the chunk does not have, and is zeroed
      // below): a load under a branch would make every later wait for an older load a wait for all
      // (the stand-in is replaced by zero when the chunk is staged, not here: using the value now
      // would wait for the load)
      const int i1 = s_i1[mo + (row >> 2)];
      g1n[k] = g1[(size_t)(i1 >= 0 ? i1 : 0) * G::S1 + (row & 3) * R1 + r1];
    }
    const int p = threadIdx.x / I3_STAGE, r = threadIdx.x - p * I3_STAGE;
    // the row index is kept raw here; taking it modulo n3 now would wait for the load at once
    i3n = uniq_row[s_u0[mo + p] + (r < s_nr[mo + p] ? r : 0)];
  };

  // registers -> LDS (buffer pair `par`) for a chunk whose operands were fetched earlier
  auto stage_chunk = [&](int par, int mo2, int cnt2) __attribute__((always_inline)) {
    float *As2 = lds + par * G::A_FLOATS, *AsT2 = As2 + G::OFF_AST;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
      const int e = threadIdx.x + k * NTHR, row = e / R1, r1 = e - row * R1;
      const float v = s_i1[mo2 + (row >> 2)] >= 0 ? g1n[k] : 0.f;  // zero rows for prefixes the chunk does not have
      As2[row * G::RS + r1] = v;
      AsT2[r1 * G::RT + row] = v;
    }
    s_i3[par][threadIdx.x / I3_STAGE][threadIdx.x % I3_STAGE] = i3n % sh.n3;
    if (wave == 0) {  // quads per prefix of the chunk, running total (scan over the first 8 lanes)
      const int q4 = (lane < TT_MP && lane < cnt2) ? (s_nr[mo2 + lane] + 3) >> 2 : 0;
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

  // The strip rows go through staging tiles that alias the H / P12 areas (not yet in use); the
  // register operands of F1 (this wavefront's 32 columns) and of T1 (the pair's 64 columns, this
  // half's r1 tiles) are then picked out of LDS.
  float breg[G::KS1][2];         // F1: B[k = r1][n = c]
  float breg2[16][G::NT1H];      // T1: B[k = c][n = r1]
  {
    float *stg = lds + G::OFF_HS;  // tile of wavefront v at v * R1 * SW: [R1][SW]
    {
      const int rsub = lane >> 3, c4 = lane & 7;  // eight rows per wavefront load
#pragma unroll
      for (int i = 0; i < R1 / 8; ++i)
        *reinterpret_cast<f32x4 *>(stg + wave * (R1 * G::SW) + (8 * i + rsub) * G::SW + 4 * c4) = sreg[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < G::KS1; ++ks)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) breg[ks][nt] = stg[wave * (R1 * G::SW) + (4 * ks + lq) * G::SW + 16 * nt + lm];
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {  // column 64*pair + 4*ks + lq lives in the tile of wavefront 2*pair + ks/8
      const int col = 4 * ks + lq, v = 2 * pair + (col >> 5);
#pragma unroll
      for (int nt = 0; nt < G::NT1H; ++nt)
        breg2[ks][nt] = stg[v * (R1 * G::SW) + (16 * (half * G::NT1H + nt) + lm) * G::SW + (col & 31)];
    }
    __syncthreads();  // the staging tiles are dead: H and P12 may be written
    // H rows of prefixes a partly filled chunk does not have are multiplied by zero core-0 rows in
    // dG2; they must hold finite numbers for that: clear H once, later chunks leave finite values
    for (int e = threadIdx.x; e < 32 * G::HS / 4; e += NTHR)
      reinterpret_cast<float4 *>(Hs)[e] = make_float4(0.f, 0.f, 0.f, 0.f);
  }

  // row batches: 32 row slots x 16 threads
  constexpr int GQ = G::CC / 16, G3Q = G::S3 / 64;  // float4 of a gradient row / a core-2 slice per thread
  int bi_p = 0, bi_ubase = 0, bi_nrow = 0, bi_last = 0;  // item record written by one thread per item
  float4 rg[GQ], r3[G3Q];
#pragma unroll
  for (int k = 0; k < GQ; ++k) rg[k] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int k = 0; k < G3Q; ++k) r3[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  int rvalid = 0;
  auto issue_batch = [&](int b, int par, int mo) __attribute__((always_inline)) {
    // global -> registers for batch b of the chunk staged in buffer pair `par` (plan entries at
    // offset `mo`); thread t serves row slot t/16
    const int total_items = s_item_off[par][TT_MP];
    const int rr = threadIdx.x >> 4, sub = threadIdx.x & 15;
    const int it = 8 * b + (rr >> 2), r = rr & 3;
    rvalid = 0;
    if (it < total_items) {
      int p = 0;
#pragma unroll
      for (int k = 1; k < TT_MP; ++k) p += (s_item_off[par][k] <= it) ? 1 : 0;
      const int r0 = 4 * (it - s_item_off[par][p]) + r;
      bi_p = p;
      bi_ubase = s_u0[mo + p] + (r0 - r);
      bi_nrow = (s_nr[mo + p] - (r0 - r)) < 4 ? (s_nr[mo + p] - (r0 - r)) : 4;
      bi_last = (r0 - r) + 4 >= s_nr[mo + p];
      if (r0 < s_nr[mo + p]) {
        const int u = s_u0[mo + p] + r0;
        const int i3 = r0 < I3_STAGE ? s_i3[par][p][r0] : uniq_row[u] % sh.n3;
        const float4 *gp = reinterpret_cast<const float4 *>(gagg + (size_t)u * G::D);
        // core 2 as stored, G3[r2][i3][0..3]: float4 r2 = sub + 16k of the row's slice
        const float4 *g3p = reinterpret_cast<const float4 *>(g3) + (size_t)sub * sh.n3 + i3;
#pragma unroll
        for (int k = 0; k < GQ; ++k) {  // float4 cc = sub + 16k of the strip: (j1, j2, 0..3)
          const int cc = sub + 16 * k;
          rg[k] = gp[(cc / G::JW) * D2 + j2base + (cc % G::JW)];
        }
#pragma unroll
        for (int k = 0; k < G3Q; ++k) r3[k] = g3p[(size_t)16 * k * sh.n3];
        rvalid = 1;
      }
    }
  };
  auto land_batch = [&]() __attribute__((always_inline)) {  // registers -> LDS
    if ((threadIdx.x & 63) == 0) {
      int *rec = s_bitem[threadIdx.x >> 6];
      rec[0] = bi_p; rec[1] = bi_ubase; rec[2] = bi_nrow; rec[3] = bi_last;
    }
    if (rvalid) {
      const int rr = threadIdx.x >> 4, sub = threadIdx.x & 15;
      float4 *gd = reinterpret_cast<float4 *>(gsm + rr * G::GS) + sub;
      float4 *g3d = reinterpret_cast<float4 *>(g3sm + rr * G::G3S) + sub;
#pragma unroll
      for (int k = 0; k < GQ; ++k) gd[16 * k] = rg[k];
#pragma unroll
      for (int k = 0; k < G3Q; ++k) g3d[16 * k] = r3[k];
    }
  };

  stage_chunk(0, 0, (seg1 - seg0) < TT_MP ? (seg1 - seg0) : TT_MP);
  int par = 0;  // buffer pair of the current chunk
  __syncthreads();
  issue_batch(0, 0, 0);  // first row batch of the first chunk

  for (int cs = seg0; cs < seg1; cs += TT_MP) {
    const int cnt = (seg1 - cs) < TT_MP ? (seg1 - cs) : TT_MP;
    const int mo = (cs - seg0) % META;  // this chunk's offset in s_q / s_i1 / s_u0 / s_nr
    __syncthreads();  // this chunk's staging is visible; previous chunk's T1 partials are consumed

    const float *As = lds + par * G::A_FLOATS, *AsT = As + G::OFF_AST;
    const bool more = cs + TT_MP < seg1, refill = mo + TT_MP == META;
    const int cnt_next = (seg1 - cs - TT_MP) < TT_MP ? (seg1 - cs - TT_MP) : TT_MP;
    const int total_items = s_item_off[par][TT_MP];
    if (more && !refill) fetch_chunk(mo + TT_MP);  // next chunk's operands, consumed right after F1

    // ---- F1: P12 of the chunk, this wavefront's 32 columns -> P12sT[p][r2][cc] -----------------
    {
      f32x4 acc[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < G::KS1; ++ks) {
        float a[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = As[(16 * mt + lm) * G::RS + 4 * ks + lq];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = MFMA(a[mt], breg[ks][nt], acc[mt][nt]);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int p = 4 * mt + lq;  // C row 4*lq + v -> prefix 4*mt + lq, j1 = v
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const int cl = 32 * wave + 16 * nt + lm, j2loc = cl / R2, r2 = cl - j2loc * R2;
#pragma unroll
          for (int v = 0; v < 4; ++v)
            P12sT[p * G::PS + r2 * G::CP + v * G::JW + j2loc] = acc[mt][nt][v];
        }
      }
    }
    land_batch();
    // All global loads of this chunk are consumed here, in one wait that F1 has mostly hidden; no
    // load is waited for while the row phase's stores are in flight.
    if (more && !refill) stage_chunk(par ^ 1, mo + TT_MP, cnt_next);
    __syncthreads();

    // ---- T3 and H over the distinct rows of the chunk, one quad (<= 4 rows of a prefix) at a time
    // Wavefronts 0-3 own one 16x16 tile of H each and walk every quad; wavefronts 4-7 own an r2 tile
    // of T3 and walk every T3_SPLIT-th quad.  The split is by output tile, not by prefix, so a
    // prefix with hundreds of rows is shared by all wavefronts and no partial sums are combined.
    // The operands of a wavefront's next quad are requested (unconditionally: the slot after a
    // batch's last quad holds older rows that are never used) before the MFMAs of the current one.
    {
      const int tw = wave & 3;
      const int hmt = tw / G::NTH, hnt = tw % G::NTH;  // H tile (wavefronts 0-3); T3: r2 tile hnt, class hmt
      const int nbatch = (total_items + 7) >> 3;
      struct Ops { float x[4], y[4]; };
      struct Ops3 { float x[G::KS3], y[G::KS3]; };
      auto walk = [&](int j0, int step, auto load_ops, auto compute) __attribute__((always_inline)) {
        for (int b = 0; b < nbatch; ++b) {
          // uniform: the next batch of a row-rich chunk is requested now and lands after this one
          if (b + 1 < nbatch) issue_batch(b + 1, par, mo);
          const int n = (total_items - 8 * b) < 8 ? (total_items - 8 * b) : 8;
          // lane l keeps the record of batch slot l % 8; a slot's fields are read with readlane
          const int4 rec = *reinterpret_cast<const int4 *>(s_bitem[lane & 7]);
          if (j0 < n) {
            auto oa = load_ops(rec, j0);
            decltype(oa) ob;
            int j = j0;
            while (true) {  // written out twice so that both operand sets stay in registers
              ob = load_ops(rec, (j + step) & 7);
              compute(rec, j, oa);
              if ((j += step) >= n) break;
              oa = load_ops(rec, (j + step) & 7);
              compute(rec, j, ob);
              if ((j += step) >= n) break;
            }
          }
          if (b + 1 < nbatch) {
            __syncthreads();  // every wavefront is done with this batch's rows
            land_batch();
            __syncthreads();
          }
        }
      };
      if (wave < 4) {  // H tile (hmt, hnt): M = cc, N = r2, K = j3, one distinct row per MFMA step
        const int hcol = 16 * hmt + lm;  // gs holds the strip's (j1, j2) columns in cc order
        f32x4 hacc = (f32x4){0.f, 0.f, 0.f, 0.f};
        walk(0, 1,
             [&](const int4 &, int j) __attribute__((always_inline)) {
               const float *gq = gsm + (j * 4) * G::GS + hcol * 4 + lq;            // the quad's four gradient rows
               const float *g3q = g3sm + (j * 4) * G::G3S + (16 * hnt + lm) * 4 + lq;  // and core-2 slices
               Ops o;
#pragma unroll
               for (int r = 0; r < 4; ++r) {
                 o.x[r] = gq[r * G::GS];
                 o.y[r] = g3q[r * G::G3S];
               }
               return o;
             },
             [&](const int4 &rec, int j, const Ops &o) __attribute__((always_inline)) {
               const int nrow = __builtin_amdgcn_readlane(rec.z, j), last = __builtin_amdgcn_readlane(rec.w, j);
#pragma unroll
               for (int r = 0; r < 4; ++r)
                 if (r < nrow) hacc = MFMA(o.x[r], o.y[r], hacc);
               if (last) {  // last quad of the prefix: H[cc = 16*hmt + 4*lq + v][r2 = 16*hnt + lm]
                 const int p = __builtin_amdgcn_readlane(rec.x, j);
#pragma unroll
                 for (int v = 0; v < 4; ++v) {
                   const int c2 = 16 * hmt + 4 * lq + v, j1 = c2 / G::JW, j2loc = c2 - j1 * G::JW;
                   Hs[(p * 4 + j1) * G::HS + j2loc * R2 + 16 * hnt + lm] = hacc[v];
                 }
                 hacc = (f32x4){0.f, 0.f, 0.f, 0.f};
               }
             });
      } else {  // T3: M = (row, j3) = lm, N = r2 tile hnt, K = cc; quads hmt, hmt + T3_SPLIT, ... (8 % T3_SPLIT == 0)
        walk(hmt, T3_SPLIT,
             [&](const int4 &rec, int j) __attribute__((always_inline)) {
               const int p = __builtin_amdgcn_readlane(rec.x, j);
               const float *ga = gsm + (j * 4 + (lm >> 2)) * G::GS + (lm & 3) + lq * 4;  // + 16*ks: cc = 4*ks + lq
               const float *pb = P12sT + p * G::PS + (16 * hnt + lm) * G::CP + lq;
               Ops3 o;
#pragma unroll
               for (int ks = 0; ks < G::KS3; ++ks) {
                 o.x[ks] = ga[16 * ks];
                 o.y[ks] = pb[4 * ks];
               }
               return o;
             },
             [&](const int4 &rec, int j, const Ops3 &o) __attribute__((always_inline)) {
               const int ubase = __builtin_amdgcn_readlane(rec.y, j), nrow = __builtin_amdgcn_readlane(rec.z, j);
               f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
               for (int ks = 0; ks < G::KS3; ++ks) acc = MFMA(o.x[ks], o.y[ks], acc);
               if (lq < nrow)
                 *reinterpret_cast<float4 *>(t3buf + ((size_t)(ubase + lq) * G::NSTRIP + strip) * G::S3 +
                                             (16 * hnt + lm) * 4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
             });
      }
    }
    __syncthreads();
    // first row batch of the NEXT chunk: requested now, landed after the next F1, so that the T1 /
    // dG2 / F1 MFMAs in between cover its latency
    if (more && !refill) issue_batch(0, par ^ 1, mo + TT_MP);

    // ---- T1 (K = the pair's 64 columns, N = this half's r1 tiles) and dG2 (N = this wavefront's 32 columns)
    {
      f32x4 acc1[2][G::NT1H];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < G::NT1H; ++nt) acc1[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        float a[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = Hs[(16 * mt + lm) * G::HS + 64 * pair + 4 * ks + lq];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < G::NT1H; ++nt) acc1[mt][nt] = MFMA(a[mt], breg2[ks][nt], acc1[mt][nt]);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < G::NT1H; ++nt)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            T1s[(pair * 32 + 16 * mt + 4 * lq + v) * R1 + 16 * (half * G::NT1H + nt) + lm] = acc1[mt][nt][v];
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      float a[G::NT1], b[2];
#pragma unroll
      for (int mt = 0; mt < G::NT1; ++mt) a[mt] = AsT[(16 * mt + lm) * G::RT + 4 * ks + lq];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) b[nt] = Hs[(4 * ks + lq) * G::HS + 32 * wave + 16 * nt + lm];
#pragma unroll
      for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc2[mt][nt] = MFMA(a[mt], b[nt], acc2[mt][nt]);
    }
    __syncthreads();
    // fold the four K-partials of T1 in pair order and store one contribution per prefix
    for (int e4 = threadIdx.x; e4 < 32 * R1 / 4; e4 += NTHR) {
      const int e = 4 * e4, row = e / R1, p = row >> 2;
      if (p < cnt) {
        const float4 x0 = *reinterpret_cast<const float4 *>(T1s + e),
                     x1 = *reinterpret_cast<const float4 *>(T1s + 32 * R1 + e),
                     x2 = *reinterpret_cast<const float4 *>(T1s + 2 * 32 * R1 + e),
                     x3 = *reinterpret_cast<const float4 *>(T1s + 3 * 32 * R1 + e);
        const float4 sum = make_float4(((x0.x + x1.x) + x2.x) + x3.x, ((x0.y + x1.y) + x2.y) + x3.y,
                                       ((x0.z + x1.z) + x2.z) + x3.z, ((x0.w + x1.w) + x2.w) + x3.w);
        *reinterpret_cast<float4 *>(t1buf + ((size_t)s_q[mo + p] * G::NSTRIP + strip) * G::S1 + (row & 3) * R1 +
                                    (e - row * R1)) = sum;
      }
    }
    if (more && refill) {  // uniform: the staged plan entries are used up, fetch the next 64
      __syncthreads();
      fetch_meta(cs + TT_MP);
      __syncthreads();
      fetch_chunk(0);
      stage_chunk(par ^ 1, 0, cnt_next);
      __syncthreads();
      issue_batch(0, par ^ 1, 0);
    }
    par ^= 1;
  }

  // dG2[r1 = 16*mt + 4*lq + v][i2][c = 32*wave + 16*nt + lm], complete for this i2 and strip
#pragma unroll
  for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float *dst = dg2 + (size_t)(16 * mt + 4 * lq + v) * sh.n2 * G::S2 + strip_col + 32 * wave + 16 * nt + lm;
        *dst = (fused && split == 1) ? fmaf(-lr, acc2[mt][nt][v], *dst) : acc2[mt][nt][v];
      }
}

// Sums the partial core-1 gradients of a split table in part order and stores the gradient, or
// applies the fused update.  One workgroup per (i2, 1024 elements of the slice); a slice no lookup
// touched is zero (or, fused, left alone).
template <bool BATCHED>
__global__ void __launch_bounds__(TT_BLOCK)
k_dg2_reduce(TTArg<BATCHED> a, int tiles) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  const int split = d.bwd_split;
  if (split <= 1 || (int)blockIdx.x >= sh.n2 * tiles) return;
  const int i2 = blockIdx.x / tiles, tile = blockIdx.x - i2 * tiles;
  const int e = (tile * TT_BLOCK + threadIdx.x) * 4;  // element of the slice [R1][S2]
  if (e >= sh.R1 * sh.S2) return;
  const int r1 = e / sh.S2, c = e - r1 * sh.S2;
  const size_t at = ((size_t)r1 * sh.n2 + i2) * sh.S2 + c, len = (size_t)sh.R1 * sh.n2 * sh.S2;
  const bool touched = d.plan.i2_seg[i2] != d.plan.i2_seg[i2 + 1];
  float *out = d.fused ? const_cast<float *>(d.g[1]) : d.dg[1];
  if (!touched) {
    if (!d.fused) *reinterpret_cast<float4 *>(out + at) = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  float4 sum = *reinterpret_cast<const float4 *>(d.plan.dg2part + at);
  for (int p = 1; p < split; ++p) {
    const float4 x = *reinterpret_cast<const float4 *>(d.plan.dg2part + p * len + at);
    sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
  }
  if (d.fused) {
    const float4 g = *reinterpret_cast<const float4 *>(out + at);
    const float lr = d.lr;
    sum = make_float4(fmaf(-lr, sum.x, g.x), fmaf(-lr, sum.y, g.y), fmaf(-lr, sum.z, g.z), fmaf(-lr, sum.w, g.w));
  }
  *reinterpret_cast<float4 *>(out + at) = sum;
}

template <int R1, int R2, int D2>
tt_status launch(const TTBatch &b, hipStream_t s) {
  using G = BwdGeom<R1, R2, D2>;
  const size_t lds = G::LDS_FLOATS * sizeof(float);
  // once per process and kernel instantiation; calls may come from several host threads
  static std::once_flag once;
  static bool configured = false;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bwd_mfma<false, R1, R2, D2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                 hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bwd_mfma<true, R1, R2, D2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
  });
  if (!configured) return TT_ERR_HIP;
  const long long blocks = tt_batch_max(b, [](const TTDev &d) {
    return (long long)d.sh.n2 * G::NSTRIP * d.bwd_split; });
  TTProfScope prof(&b.host[0].plan, TT_KERNEL_BWD_CONTRACT, s);
  if (b.dev)
    hipLaunchKernelGGL((k_bwd_mfma<true, R1, R2, D2>), dim3((unsigned)blocks, (unsigned)b.T),
                       dim3(NTHR), lds, s, TTArg<true>{b.dev});
  else
    hipLaunchKernelGGL((k_bwd_mfma<false, R1, R2, D2>), dim3((unsigned)blocks), dim3(NTHR), lds, s,
                       TTArg<false>{b.host[0]});
  if (tt_batch_max(b, [](const TTDev &d) { return (long long)d.bwd_split; }) > 1) {
    const int tiles = tt_ceil_div((long long)R1 * G::S2, TT_BLOCK * 4);
    const long long n2max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n2; });
    TT_LAUNCH(k_dg2_reduce, n2max * tiles, TT_BLOCK, 0, s, b, tiles);
  }
  return tt_launch_status();
}

}  // namespace

int ttk_mfma_strips(const TTShape &sh) {
  return ttk_forward_mfma_supported(sh) ? (sh.d2 * sh.R2) / 256 : 1;
}

int ttk_bwd_split(const TTShape &sh) {
  if (!ttk_forward_mfma_supported(sh)) return 1;
  const int wgs = sh.n2 * ttk_mfma_strips(sh);
  if (wgs >= 128) return 1;
  const int s = 256 / wgs;
  return s > TT_BWD_MAX_SPLIT ? TT_BWD_MAX_SPLIT : s;
}

tt_status ttk_backward_mfma(const TTBatch &b, hipStream_t s) {
  if (b.host[0].sh.R1 == 32) return launch<32, 32, 8>(b, s);
  return launch<64, 64, 8>(b, s);
}
