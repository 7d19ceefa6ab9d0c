// MFMA backward contractions for the TT embedding bag (paper Section III-D backward equation,
// after the in-advance gradient aggregation of Section III-E), gfx950.
//
// One workgroup owns one (i2, strip) of the core-1 slice G2[:, i2, :, :], where a strip is ALL j2
// and a block of 16 values of r2 (128 columns c = (j2, r2l)), and walks the distinct prefixes
// (i1, i2) of the batch in chunks of TT_MP = 8.  With g = the merged output gradient of a distinct
// row, per chunk it forms
//   F1  P12[(p,j1)][c]   = sum_r1 G1[i1_p][j1][r1] G2[r1][i2][c]                 (recomputed, LDS)
//   T3  t3[u][r2][j3]    = sum_{j1,j2} P12[p][j1][j2][r2] g[u][j1][j2][j3]       (per row, r2 in strip)
//   H   H[p][j1][c]      = sum_{rows u of p} sum_j3 g[u][j1][j2][j3] G3[r2][i3_u][j3]
//   T1  t1[p][j1][r1]    = sum_{c in strip} H[p][j1][c] G2[r1][i2][c]             (per prefix)
//   dG2[r1][i2][c]      += sum_{p in chunk} sum_j1 G1[i1_p][j1][r1] H[p][j1][c]
// all on v_mfma_f32_16x16x4_f32.  Cutting the slice by r2 (not by j2) makes t3 complete inside one
// strip -- it sums over j1 and j2 only -- so every distinct row's core-2 contribution is written
// once, and a strip needs only its own 16 of the R2 rows of each core-2 slice.  dG2 stays in
// accumulator registers over all chunks of the i2 and is written once (no atomics); t1 is a
// per-prefix contribution per strip; sorted segmented sums fold t3 / t1 into dG3 / dG1 afterwards.
//
// A workgroup is four wavefronts and uses under 80 KB of LDS, so that TWO workgroups share a
// compute unit: while one waits for memory or stages operands, the other's MFMAs keep the matrix
// cores busy (a workgroup alternates between phases that are all-MFMA and phases that are all
// staging, so one alone leaves the matrix cores idle about half the time).
//   F1        wavefront w owns columns [32w, 32w + 32) of the strip, both 16-row tiles;
//   T1        wavefront w owns an r1 tile (R1 = 64) or a (row tile, r1 tile) pair (R1 = 32), all
//             128 columns as K: no partial sums cross wavefronts;
//   dG2       wavefront w owns columns [32w, 32w + 32), all r1;
//   row phase wavefronts 0-1 accumulate the two H tiles of a prefix, wavefronts 2-3 form the T3
//             tiles of alternate row quads: four MFMAs per quad for every wavefront.
// Both register views of the strip (B of F1: lanes along c; B of T1: lanes along r1) are picked
// once per workgroup out of an LDS staging tile.
//
// MFMA operand layout (D = A[16x4] * B[4x16] + C): lane l supplies A[m = l%16][k = l/16] and
// B[k = l/16][n = l%16] and holds C[m = 4*(l/16) + v][n = l%16] in component v.
#include <mutex>

#include "tt_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)
constexpr int NTHR = 256;   // threads per workgroup
constexpr int META = 64;    // prefixes whose plan entries are fetched into LDS in one go (8 chunks)
constexpr int RB = 16;      // r2 values per strip
constexpr int NROW = 32;    // distinct rows per batch of the row phase (8 quads)

template <int R1, int R2>
struct BwdGeom {
  static constexpr int D2 = 8;
  static constexpr int NSB = R2 / RB;      // strips per core-1 slice
  static constexpr int SC = D2 * RB;       // columns per strip (128)
  static constexpr int S2 = D2 * R2;
  static constexpr int D = 128, S1 = 4 * R1, S3 = R2 * 4;
  // LDS row strides.  A 64-lane read is served in two halves (lanes 0-31: lq = 0,1); the strides put
  // the 32 lanes of a half on 32 different banks for the access named first.
  static constexpr int RS = R1 + 2;        // As  [32 (p,j1)][R1]   F1 A operand: row = lm, +lq (dG2 A operand: row = lq, +lm, 2-way)
  static constexpr int PS = 32 * RB + 16;  // P12 [p][cc = 32][r2l = 16]  F1 store / T3 B operand: 16*lq + lm
  static constexpr int HR = SC + 2;        // Hs  [32 (p,j1)][128 c]      T1 A operand: row = lm, +lq (dG2 B operand 2-way)
  static constexpr int GS = D + 8;         // gs  [32 rows][(cc, j3)]     T3 A operand: row = lm/4, 4*lq + lm%4
  static constexpr int G3S = RB * 4;       // g3s [32 rows][(r2l, j3)]
  static constexpr int SW = SC + 4;        // strip staging tile [R1][128 c] (float4 rows)
  static constexpr int KS1 = R1 / 4;       // k steps of F1
  static constexpr int NT1 = R1 / 16;      // r1 tiles
  static constexpr int T1_MT = NT1 == 4 ? 2 : 1;  // row tiles of T1 per wavefront
  static constexpr int A_FLOATS = 32 * RS;        // one core-0 tile; two of them: current chunk / next chunk
  static constexpr int OFF_P12 = 2 * A_FLOATS;
  static constexpr int OFF_HS = OFF_P12 + TT_MP * PS;
  static constexpr int OFF_GS = OFF_HS + 32 * HR;
  static constexpr int OFF_G3S = OFF_GS + NROW * GS;
  static constexpr size_t LDS_FLOATS = (size_t)OFF_G3S + (NROW + 8) * G3S;  // spare rows: operand prefetch reads up to two groups of four rows ahead
  static constexpr int GPT = (32 * R1) / NTHR;  // core-0 tile elements per thread
  static_assert(R2 % RB == 0 && (R1 == 32 || R1 == 64) && TT_MP == 8, "shape");
  static_assert(R1 * SW <= TT_MP * PS + 32 * HR + NROW * GS, "the strip staging tile aliases the P12 / H / row areas");
  static_assert(LDS_FLOATS * 4 + 2048 <= 80 * 1024, "two workgroups per compute unit");
  static_assert(OFF_P12 % 4 == 0 && OFF_GS % 4 == 0 && OFF_G3S % 4 == 0 && GS % 4 == 0, "float4 accesses");
};

template <bool BATCHED, int R1, int R2>
__global__ void __launch_bounds__(NTHR, 2)
k_bwd_mfma(TTArg<BATCHED> a) {
  const TTDev &d = a.get();
  const TTShape &sh = d.sh;
  using G = BwdGeom<R1, R2>;
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
  extern __shared__ float lds[];
  float *P12s = lds + G::OFF_P12, *Hs = lds + G::OFF_HS;  // core-0 tiles: lds + par * A_FLOATS
  float *gsm = lds + G::OFF_GS, *g3sm = lds + G::OFF_G3S;
  // per row slot of the current batch: x = prefix | rows of the item that starts here << 4 (0: none
  // starts here) | item is the prefix's last << 8 | row is the prefix's last << 9; y = the row's slot
  __shared__ __align__(8) int s_brow[NROW][2];
  __shared__ int s_q[META], s_i1[META], s_u0[META], s_nr[META];

  // workgroup = (i2, strip, part): with split > 1 the chunks of one (i2, strip) are dealt in
  // contiguous runs to `split` workgroups, each of which leaves a partial core-1 gradient
  // Workgroup index = ((i2 / 8) * (strips * split) + (strip, part)) * 8 + i2 % 8.  Workgroups are
  // dealt to the 8 XCDs round-robin, so all strips and parts of one i2 run on XCD i2 % 8, close in
  // time, and find the merged gradients and plan entries of that i2's rows in its L2; and the
  // i2 values are started in increasing order (with Zipf ranks as row numbers the hot prefixes, whose
  // workgroups run longest, are the ones with small i2).
  const int split = d.bwd_split, nsub = G::NSB * split;
  const int i2 = (int)(blockIdx.x / (8 * nsub)) * 8 + (int)(blockIdx.x & 7), sub = (int)(blockIdx.x >> 3) % nsub;
  if (i2 >= sh.n2) return;  // padding of the last group of 8, or a table of the batch with fewer i2 values
  const int sblk = sub / split, part = sub - sblk * split;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lm = lane & 15, lq = lane >> 4;
  // element (r1, c = (j2, r2l)) of the strip sits at strip_col + r1 * r1_stride + j2 * R2 + r2l
  const size_t strip_col = (size_t)i2 * G::S2 + sblk * RB;
  const size_t r1_stride = (size_t)sh.n2 * G::S2;

  // The strip is read from memory once, as 64-byte pieces (one (r1, j2): 16 r2 values), float4 per
  // lane.  The loads depend on the workgroup index only and are requested before the plan is looked
  // at, so that their latency overlaps the chain of dependent plan loads.
  f32x4 sreg[R1 / 8];
  {
    const int rsub = threadIdx.x >> 5, s = threadIdx.x & 31;  // 8 rows per pass, 32 float4 per row
#pragma unroll
    for (int i = 0; i < R1 / 8; ++i)
      sreg[i] = *reinterpret_cast<const f32x4 *>(g2 + (size_t)(8 * i + rsub) * r1_stride + strip_col + (s >> 2) * R2 + 4 * (s & 3));
  }
  int seg0 = i2_seg[i2], seg1 = i2_seg[i2 + 1];
  const bool touched = seg0 != seg1;
  if (split > 1) {
    const int nch = (seg1 - seg0 + TT_MP - 1) / TT_MP, per = (nch + split - 1) / split;
    const int c0 = part * per, c1 = (c0 + per) < nch ? (c0 + per) : nch;
    const int lo = seg0 + c0 * TT_MP, hi = seg0 + c1 * TT_MP;
    seg1 = c0 < c1 ? (hi < seg1 ? hi : seg1) : seg0;
    seg0 = c0 < c1 ? lo : seg0;
    dg2 = d.plan.dg2part + (size_t)part * R1 * r1_stride;  // partial gradients have the shape of core 1
  }

  if (seg0 == seg1) {  // uniform: no prefix for this workgroup, its gradient strip is zero
    if ((fused && split == 1) || (split > 1 && !touched)) return;  // nothing will read it
    for (int e = threadIdx.x; e < R1 * G::SC; e += NTHR) {
      const int r1 = e / G::SC, c = e - r1 * G::SC;
      dg2[(size_t)r1 * r1_stride + strip_col + (c >> 4) * R2 + (c & 15)] = 0.f;
    }
    return;
  }

  // dG2[m = r1][n = c], this wavefront's 32 columns, persistent over the chunks
  f32x4 acc2[G::NT1][2];
#pragma unroll
  for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) acc2[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Core-0 rows of the NEXT chunk are fetched into registers while the current chunk computes.
  float g1n[G::GPT];
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
    for (int k = 0; k < G::GPT; ++k) {
      const int e = threadIdx.x + k * NTHR, row = e / R1, r1 = e - row * R1;
      // unconditional (slice 0 stands in for a prefix the chunk does not have; it is replaced by
      // zero when the chunk is staged, so that no load sits under a branch)
      const int i1 = s_i1[mo + (row >> 2)];
      g1n[k] = g1[(size_t)(i1 >= 0 ? i1 : 0) * G::S1 + (row & 3) * R1 + r1];
    }
  };
  auto stage_chunk = [&](int par, int mo) __attribute__((always_inline)) {  // registers -> core-0 tile `par`
    float *As2 = lds + par * G::A_FLOATS;
#pragma unroll
    for (int k = 0; k < G::GPT; ++k) {
      const int e = threadIdx.x + k * NTHR, row = e / R1, r1 = e - row * R1;
      As2[row * G::RS + r1] = s_i1[mo + (row >> 2)] >= 0 ? g1n[k] : 0.f;  // zero rows for prefixes the chunk does not have
    }
  };

  // Row batches: the distinct rows of a chunk, prefix after prefix, are cut into batches of 32; an
  // ITEM is a run of at most 4 rows of one prefix inside a batch (it starts at every fourth row of a
  // prefix and at a batch boundary).  Thread t serves row slot t/8 of the batch: a float4 of the
  // merged gradient row per 8 columns, and the strip's 16 rows of the core-2 slice (one float4 each).
  int bi_x = 0, bi_y = 0;
  float4 rg[4], r3[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) rg[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  r3[0] = r3[1] = make_float4(0.f, 0.f, 0.f, 0.f);
  int rvalid = 0;
  auto chunk_rows = [&](int mo) __attribute__((always_inline)) {  // distinct rows of the chunk
    int tot = 0;
#pragma unroll
    for (int k = 0; k < TT_MP; ++k) tot += s_nr[mo + k];
    return tot;
  };
  // The row of the table behind row slot `rr` of batch b (its i3 selects the core-2 slice): loaded
  // one step before the batch's operands are requested, so that a batch costs one memory round
  // trip, not two dependent ones.  Rows past the chunk's end read slot 0 (never used).
  auto row_slot = [&](int R, int mo, int &p, int &before, int &run) __attribute__((always_inline)) {
    p = 0; before = 0; run = 0;  // prefix that holds row R of the chunk, rows before that prefix, rows of the chunk
#pragma unroll
    for (int k = 0; k < TT_MP; ++k) {
      if (run <= R) { p = k; before = run; }
      run += s_nr[mo + k];
    }
  };
  auto fetch_row_id = [&](int b, int mo) __attribute__((always_inline)) {
    int p, before, run;
    const int R = NROW * b + (threadIdx.x >> 3);
    row_slot(R, mo, p, before, run);
    return uniq_row[R < run ? s_u0[mo + p] + (R - before) : 0];
  };
  auto issue_batch = [&](int b, int mo, int row_id) __attribute__((always_inline)) {
    // global -> registers for batch b of the chunk whose plan entries sit at offset `mo`
    const int rr = threadIdx.x >> 3, sub = threadIdx.x & 7;
    const int R = NROW * b + rr;  // row of the chunk
    int p, before, run;
    row_slot(R, mo, p, before, run);
    rvalid = 0;
    bi_x = 0; bi_y = 0;
    if (R < run) {
      const int nr = s_nr[mo + p], r0 = R - before, u = s_u0[mo + p] + r0;
      int nrow = 0;
      if ((r0 & 3) == 0 || rr == 0) {  // an item starts here
        nrow = 4 - (r0 & 3);
        nrow = nrow < nr - r0 ? nrow : nr - r0;
        nrow = nrow < NROW - rr ? nrow : NROW - rr;
      }
      bi_x = p | (nrow << 4) | ((r0 + nrow == nr) ? 256 : 0) | ((r0 + 1 == nr) ? 512 : 0);
      bi_y = u;
      const int i3 = row_id % sh.n3;
      const float4 *gp = reinterpret_cast<const float4 *>(gagg + (size_t)u * G::D);
      // core 2 as stored, G3[r2][i3][0..3]: one float4 per r2 of the strip
      const float4 *g3p = reinterpret_cast<const float4 *>(g3) + (size_t)(sblk * RB + sub) * sh.n3 + i3;
#pragma unroll
      for (int k = 0; k < 4; ++k) rg[k] = gp[sub + 8 * k];
#pragma unroll
      for (int k = 0; k < 2; ++k) r3[k] = g3p[(size_t)8 * k * sh.n3];
      rvalid = 1;
    }
  };
  auto land_batch = [&]() __attribute__((always_inline)) {  // registers -> LDS
    const int rr = threadIdx.x >> 3, sub = threadIdx.x & 7;
    if (sub == 0) { s_brow[rr][0] = bi_x; s_brow[rr][1] = bi_y; }
    if (rvalid) {
      float4 *gd = reinterpret_cast<float4 *>(gsm + rr * G::GS) + sub;
      float4 *g3d = reinterpret_cast<float4 *>(g3sm + rr * G::G3S) + sub;
#pragma unroll
      for (int k = 0; k < 4; ++k) gd[8 * k] = rg[k];
#pragma unroll
      for (int k = 0; k < 2; ++k) g3d[8 * k] = r3[k];
    }
  };

  fetch_meta(seg0);
  __syncthreads();
  fetch_chunk(0);

  // The strip rows go through a staging tile that aliases the P12 / H / row areas (not yet in use);
  // the register operands of F1 (this wavefront's 32 columns) and of T1 (this wavefront's r1 tile,
  // all columns) are then picked out of LDS.
  float breg[G::KS1][2];   // F1: B[k = r1][n = c]
  float breg2[32];         // T1: B[k = c][n = r1]
  const int t1_nt = G::NT1 == 4 ? wave : (wave & 1);  // r1 tile of this wavefront in T1
  {
    float *stg = lds + G::OFF_P12;  // [R1][SW]
    {
      const int rsub = threadIdx.x >> 5, s = threadIdx.x & 31;
#pragma unroll
      for (int i = 0; i < R1 / 8; ++i)
        *reinterpret_cast<f32x4 *>(stg + (8 * i + rsub) * G::SW + 4 * s) = sreg[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < G::KS1; ++ks)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) breg[ks][nt] = stg[(4 * ks + lq) * G::SW + 32 * wave + 16 * nt + lm];
#pragma unroll
    for (int ks = 0; ks < 32; ++ks) breg2[ks] = stg[(16 * t1_nt + lm) * G::SW + 4 * ks + lq];
    __syncthreads();  // the staging tile is dead: P12, H and the row areas may be written
    // H rows of prefixes a partly filled chunk does not have are multiplied by zero core-0 rows in
    // dG2; they must hold finite numbers for that: clear H once, later chunks leave finite values
    for (int e = threadIdx.x; e < 32 * G::HR; e += NTHR) Hs[e] = 0.f;
  }

  stage_chunk(0, 0);
  issue_batch(0, 0, fetch_row_id(0, 0));  // first row batch of the first chunk
  int par = 0;        // core-0 tile of the current chunk

  for (int cs = seg0; cs < seg1; cs += TT_MP) {
    const int cnt = (seg1 - cs) < TT_MP ? (seg1 - cs) : TT_MP;
    const int mo = (cs - seg0) % META;  // this chunk's offset in s_q / s_i1 / s_u0 / s_nr
    const bool more = cs + TT_MP < seg1, refill = mo + TT_MP == META;
    __syncthreads();  // this chunk's core-0 tile is visible; the previous chunk's readers of H and of the other tile are done
    const float *As = lds + par * G::A_FLOATS;
    const int total_rows = chunk_rows(mo);
    if (more && !refill) fetch_chunk(mo + TT_MP);  // next chunk's core-0 rows, staged into the other tile after the row phase
    // row ids for the second batch of this chunk and the first batch of the next one
    int id_next_batch = fetch_row_id(1, mo);
    const int id_next_chunk = (more && !refill) ? fetch_row_id(0, mo + TT_MP) : 0;

    // ---- F1: P12 of the chunk, this wavefront's 32 columns -> P12s[p][cc = (j1, j2)][r2l] ----------
    {
      f32x4 acc[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < G::KS1; ++ks) {
        float av[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) av[mt] = As[(16 * mt + lm) * G::RS + 4 * ks + lq];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = MFMA(av[mt], breg[ks][nt], acc[mt][nt]);
      }
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int p = 4 * mt + lq;  // C row 4*lq + v -> prefix 4*mt + lq, j1 = v
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const int j2 = 2 * wave + nt;  // column 32*wave + 16*nt + lm = (j2, r2l = lm)
#pragma unroll
          for (int v = 0; v < 4; ++v) P12s[p * G::PS + (v * 8 + j2) * RB + lm] = acc[mt][nt][v];
        }
      }
    }
    land_batch();
    __syncthreads();

    // ---- T3 and H over the distinct rows of the chunk, one quad (<= 4 rows of a prefix) at a time
    // Wavefronts 0-1 own one 16x16 tile of H each (cc tile = wavefront) and walk every quad;
    // wavefronts 2-3 form the T3 tile of every other quad.  The split is by output tile, so a prefix
    // with hundreds of rows is shared by all wavefronts and no partial sums are combined.
    {
      const int nbatch = (total_rows + NROW - 1) / NROW;
      f32x4 hacc = (f32x4){0.f, 0.f, 0.f, 0.f};
      for (int b = 0; b < nbatch; ++b) {
        // uniform: the next batch of a row-rich chunk is requested now and lands after this one
        if (b + 1 < nbatch) {
          issue_batch(b + 1, mo, id_next_batch);
          id_next_batch = fetch_row_id(b + 2, mo);
        }
        const int n = (total_rows - NROW * b) < NROW ? (total_rows - NROW * b) : NROW;
        // lane l keeps the record of row slot l % 32; a slot's fields are read with readlane
        const int2 rec = *reinterpret_cast<const int2 *>(s_brow[lane & (NROW - 1)]);
        // The batch is a run of items (<= 4 rows of one prefix each): the item at row slot rr has
        // `nrow` rows and the next one starts at rr + nrow.  Both loops below are written for few
        // instructions per row -- with one or two wavefronts per SIMD the row phase is bound by
        // instruction issue, not by the matrix cores.
        if (wave < 2) {  // H tile `wave`: M = cc, N = r2l, K = j3, one distinct row per MFMA
          // The operands of the next item are requested before the MFMAs of the current one (an item's
          // four row slots are always read; slots past its rows belong to later rows and are not used).
          const float *gq = gsm + (16 * wave + lm) * 4 + lq;
          const float *g3q = g3sm + lm * 4 + lq;
          struct Ops { float x[4], y[4]; };
          auto load_ops = [&](int r0) __attribute__((always_inline)) {
            Ops o;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              o.x[r] = gq[(r0 + r) * G::GS];
              o.y[r] = g3q[(r0 + r) * G::G3S];
            }
            return o;
          };
          auto compute = [&](int f, const Ops &o) __attribute__((always_inline)) {
            const int nrow = (f >> 4) & 15;
            hacc = MFMA(o.x[0], o.y[0], hacc);
            if (nrow > 1) {  // uniform
              hacc = MFMA(o.x[1], o.y[1], hacc);
              if (nrow > 2) {
                hacc = MFMA(o.x[2], o.y[2], hacc);
                if (nrow > 3) hacc = MFMA(o.x[3], o.y[3], hacc);
              }
            }
            if (f & 256) {  // the prefix ends with this item: H[cc = 16*wave + 4*lq + v][r2l = lm]
              float *hp = Hs + ((f & 15) * 4 + 2 * wave + (lq >> 1)) * G::HR + (4 * (lq & 1)) * RB + lm;
#pragma unroll
              for (int v = 0; v < 4; ++v) hp[v * RB] = hacc[v];  // cc = (j1 = 2*wave + lq/2, j2 = 4*(lq%2) + v)
              hacc = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
          };
          int rr = 0, f = __builtin_amdgcn_readlane(rec.x, 0);
          Ops oa = load_ops(0), ob;
          while (true) {  // written out twice so that both operand sets stay in registers
            int rn = rr + ((f >> 4) & 15);
            int fn = __builtin_amdgcn_readlane(rec.x, rn & (NROW - 1));
            ob = load_ops(rn);
            compute(f, oa);
            if (rn >= n) break;
            rr = rn + ((fn >> 4) & 15);
            f = __builtin_amdgcn_readlane(rec.x, rr & (NROW - 1));
            oa = load_ops(rr);
            compute(fn, ob);
            if (rr >= n) break;
          }
        } else {  // T3: M = (row, j3) = lm, N = r2l, K = cc; wavefront 2 takes the even items, 3 the odd ones
          struct Ops3 { float a[8], b[8]; };
          auto load_ops = [&](int rr, int f) __attribute__((always_inline)) {
            const float *ga = gsm + (rr + (lm >> 2)) * G::GS + (lm & 3) + lq * 4;  // + 16*ks: cc = 4*ks + lq
            const float *pb = P12s + (f & 15) * G::PS + lq * RB + lm;               // + 64*ks
            Ops3 o;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
              o.a[ks] = ga[16 * ks];
              o.b[ks] = pb[4 * RB * ks];
            }
            return o;
          };
          auto compute = [&](int rr, int f, const Ops3 &o) __attribute__((always_inline)) {
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f}, accb = (f32x4){0.f, 0.f, 0.f, 0.f};  // two chains of four
#pragma unroll
            for (int ks = 0; ks < 8; ks += 2) {
              acc = MFMA(o.a[ks], o.b[ks], acc);
              accb = MFMA(o.a[ks + 1], o.b[ks + 1], accb);
            }
            const int ubase = __builtin_amdgcn_readlane(rec.y, rr);
            if (lq < ((f >> 4) & 15))
              *reinterpret_cast<float4 *>(t3buf + (size_t)(ubase + lq) * G::S3 + (sblk * RB + lm) * 4) =
                  make_float4(acc[0] + accb[0], acc[1] + accb[1], acc[2] + accb[2], acc[3] + accb[3]);
          };
          // (row slot, record) of this wavefront's next item at or after row slot rr, skipping `skip` items
          auto next_item = [&](int &rr, int &f, int skip) __attribute__((always_inline)) {
            f = __builtin_amdgcn_readlane(rec.x, rr & (NROW - 1));
            for (int k = 0; k < skip && rr < n; ++k) {
              rr += (f >> 4) & 15;
              f = __builtin_amdgcn_readlane(rec.x, rr & (NROW - 1));
            }
          };
          int rr = 0, f;
          next_item(rr, f, wave - 2);
          if (rr < n) {
            Ops3 oa = load_ops(rr, f), ob;
            while (true) {  // written out twice so that both operand sets stay in registers
              int rn = rr, fn;
              next_item(rn, fn, 2);
              if (rn < n) ob = load_ops(rn, fn);
              compute(rr, f, oa);
              if (rn >= n) break;
              rr = rn;
              next_item(rr, f, 2);
              if (rr < n) oa = load_ops(rr, f);
              compute(rn, fn, ob);
              if (rr >= n) break;
            }
          }
        }
        if (b + 1 < nbatch) {
          __syncthreads();  // every wavefront is done with this batch's rows
          land_batch();
          __syncthreads();
        }
      }
    }
    __syncthreads();  // H of the chunk is complete; P12 and the row areas are free
    // first row batch of the NEXT chunk: requested now, landed after the next F1, so that the T1 /
    // dG2 / F1 MFMAs in between cover its latency
    if (more && !refill) {
      issue_batch(0, mo + TT_MP, id_next_chunk);
      stage_chunk(par ^ 1, mo + TT_MP);  // the other core-0 tile was last read by the previous chunk
    }

    // ---- T1: this wavefront's tile(s) [16 (p,j1)] x [16 r1], K = the strip's 128 columns ------------
    {
      f32x4 acc1[G::T1_MT];
#pragma unroll
      for (int mt = 0; mt < G::T1_MT; ++mt) acc1[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const int mt0 = G::NT1 == 4 ? 0 : (wave >> 1);
#pragma unroll
      for (int ks = 0; ks < 32; ++ks) {
        float av[G::T1_MT];
#pragma unroll
        for (int mt = 0; mt < G::T1_MT; ++mt) av[mt] = Hs[(16 * (mt0 + mt) + lm) * G::HR + 4 * ks + lq];
#pragma unroll
        for (int mt = 0; mt < G::T1_MT; ++mt) acc1[mt] = MFMA(av[mt], breg2[ks], acc1[mt]);
      }
      // C[m = (p, j1) = 4*lq + v][n = r1 = 16*t1_nt + lm]: one contribution per prefix and strip
#pragma unroll
      for (int mt = 0; mt < G::T1_MT; ++mt) {
        const int p = 4 * (mt0 + mt) + lq;
        if (p < cnt) {
          float *dst = t1buf + ((size_t)s_q[mo + p] * G::NSB + sblk) * G::S1 + 16 * t1_nt + lm;
#pragma unroll
          for (int v = 0; v < 4; ++v) dst[v * R1] = acc1[mt][v];
        }
      }
    }
    // ---- dG2 += G1^T H: M = r1, N = this wavefront's 32 columns, K = the chunk's 32 (p, j1) rows ----
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      float av[G::NT1], bv[2];
#pragma unroll
      for (int mt = 0; mt < G::NT1; ++mt) av[mt] = As[(4 * ks + lq) * G::RS + 16 * mt + lm];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) bv[nt] = Hs[(4 * ks + lq) * G::HR + 32 * wave + 16 * nt + lm];
#pragma unroll
      for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc2[mt][nt] = MFMA(av[mt], bv[nt], acc2[mt][nt]);
    }
    if (more && refill) {  // uniform: the staged plan entries are used up, fetch the next 64
      __syncthreads();  // every reader of the plan entries is done
      fetch_meta(cs + TT_MP);
      __syncthreads();
      fetch_chunk(0);
      stage_chunk(par ^ 1, 0);
      issue_batch(0, 0, fetch_row_id(0, 0));
    }
    par ^= 1;
  }

  // dG2[r1 = 16*mt + 4*lq + v][i2][c = 32*wave + 16*nt + lm], complete for this i2 and strip.  With
  // the fused update every old core element is requested before the first store (the core may alias
  // nothing here, but the compiler cannot know: load / store pairs would each wait for memory).
  float *dbase = dg2 + (size_t)(4 * lq) * r1_stride + strip_col + (2 * wave) * R2 + lm;
  if (fused && split == 1) {
    float old[G::NT1][2][4];
#pragma unroll
    for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) old[mt][nt][v] = dbase[(size_t)(16 * mt + v) * r1_stride + nt * R2];
#pragma unroll
    for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          dbase[(size_t)(16 * mt + v) * r1_stride + nt * R2] = fmaf(-lr, acc2[mt][nt][v], old[mt][nt][v]);
  } else {
#pragma unroll
    for (int mt = 0; mt < G::NT1; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) dbase[(size_t)(16 * mt + v) * r1_stride + nt * R2] = acc2[mt][nt][v];
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

template <int R1, int R2>
tt_status launch(const TTBatch &b, hipStream_t s) {
  using G = BwdGeom<R1, R2>;
  const size_t lds = G::LDS_FLOATS * sizeof(float);
  // once per process and kernel instantiation; calls may come from several host threads
  static std::once_flag once;
  static bool configured = false;
  std::call_once(once, [&] {
    configured = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bwd_mfma<false, R1, R2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                 hipFuncSetAttribute(reinterpret_cast<const void *>(&k_bwd_mfma<true, R1, R2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
  });
  if (!configured) return TT_ERR_HIP;
  const long long blocks = tt_batch_max(b, [](const TTDev &d) {
    return (long long)((d.sh.n2 + 7) & ~7) * G::NSB * d.bwd_split; });
  {
    // the contraction kernel alone, timed by its own begin and end stamps when a profile object asks
    TTProfScope prof(&b.host[0].plan, TT_KERNEL_BWD_CONTRACT, s, false);
    if (b.dev)
      hipExtLaunchKernelGGL((k_bwd_mfma<true, R1, R2>), dim3((unsigned)blocks, (unsigned)b.T),
                            dim3(NTHR), lds, s, prof.start(), prof.stop(), 0, TTArg<true>{b.dev});
    else
      hipExtLaunchKernelGGL((k_bwd_mfma<false, R1, R2>), dim3((unsigned)blocks), dim3(NTHR), lds, s,
                            prof.start(), prof.stop(), 0, TTArg<false>{b.host[0]});
  }
  if (tt_batch_max(b, [](const TTDev &d) { return (long long)d.bwd_split; }) > 1) {
    const int tiles = tt_ceil_div((long long)R1 * G::S2, TT_BLOCK * 4);
    const long long n2max = tt_batch_max(b, [](const TTDev &d) { return (long long)d.sh.n2; });
    TT_LAUNCH(k_dg2_reduce, n2max * tiles, TT_BLOCK, 0, s, b, tiles);
  }
  return tt_launch_status();
}

}  // namespace

int ttk_mfma_strips(const TTShape &sh) {
  return ttk_forward_mfma_supported(sh) ? sh.R2 / RB : 1;
}

#ifndef TT_BWD_SPLIT_BELOW
#define TT_BWD_SPLIT_BELOW 256
#endif
#ifndef TT_BWD_SPLIT_TARGET
#define TT_BWD_SPLIT_TARGET 512
#endif
int ttk_bwd_split(const TTShape &sh) {
  if (!ttk_forward_mfma_supported(sh)) return 1;
  // two workgroups fit on each of the 256 compute units: a table with fewer than 256 (i2, strip)
  // pairs deals the chunks of each pair to several workgroups
  const int wgs = sh.n2 * ttk_mfma_strips(sh);
  if (wgs >= TT_BWD_SPLIT_BELOW) return 1;
  const int s = TT_BWD_SPLIT_TARGET / wgs;
  return s > TT_BWD_MAX_SPLIT ? TT_BWD_MAX_SPLIT : (s < 1 ? 1 : s);
}

tt_status ttk_backward_mfma(const TTBatch &b, hipStream_t s) {
  if (b.host[0].sh.R1 == 32) return launch<32, 32>(b, s);
  return launch<64, 64>(b, s);
}
