// Sanitizer harness of the CPU emulation: runs the C ABI of the library, single-table and batched,
// on a few small tables with seeded inputs and checks that the batched calls give bit-for-bit the
// single-table results.  Built with AddressSanitizer + UBSan (or MemorySanitizer / ThreadSanitizer,
// see build.py), so every out-of-bounds, misaligned or racing LDS access of a kernel is reported.
// usage: harness <mfma | plain | unaligned | wide | keys31 | cfg5like> [planned: 1 | 0] [bags for cfg5like]
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#include <math.h>
#include <vector>
#include "tt_emb.h"

// regions the kernels must never touch (host structs of the C ABI): poisoned while a launch runs
namespace emu { void host_only(const void *p, size_t n); void host_only_release(const void *p); }

static int g_off = 0;  // floats by which core and gradient pointers are shifted off their alignment
static uint64_t rs = 88172645463325252ull;
static uint32_t rnd() { rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17; return (uint32_t)(rs >> 11); }
static float rndf() { return ((int)(rnd() % 2001) - 1000) / 1000.0f; }

struct Tab {
  tt_table t;
  std::vector<float> core[3], core0[3];
  std::vector<int64_t> idx, off;
  std::vector<float> grad;
  int64_t nnz, bags;
  int D;
};

static void *amalloc(size_t n) { void *p = nullptr; if (posix_memalign(&p, 256, n ? n : 256)) abort();
#ifdef EMU_MSAN
  return p;  // left uninitialised on purpose: MemorySanitizer tracks reads of it
#endif
  { const char *e = getenv("EMU_FILL"); memset(p, e ? (int)strtol(e, 0, 0) : 0xA5, n); } return p; }

static Tab make_tab(const int n[3], const int d[3], int R1, int R2, int bags, int maxlen, int64_t num_rows) {
  Tab T;
  memset(&T.t, 0, sizeof(T.t));
  T.t.num_rows = num_rows;
  for (int k = 0; k < 3; ++k) { T.t.n[k] = n[k]; T.t.d[k] = d[k]; }
  T.t.r[0] = 1; T.t.r[1] = R1; T.t.r[2] = R2; T.t.r[3] = 1;
  for (int k = 0; k < 3; ++k) {
    size_t len = (size_t)T.t.r[k] * n[k] * d[k] * T.t.r[k + 1];
    T.core[k].resize(len + 1);
    for (auto &x : T.core[k]) x = rndf() * 0.3f;
    T.core0[k] = T.core[k];
  }
  T.D = d[0] * d[1] * d[2];
  T.bags = bags;
  T.off.push_back(0);
  for (int b = 0; b < bags; ++b) {
    int len = maxlen <= 1 ? 1 : (int)(rnd() % (maxlen + 1));
    for (int l = 0; l < len; ++l) {
      // skewed: small rows are hot
      // roughly Zipf(1): rank = N^u, u uniform
      double u = (rnd() % 1000003) / 1000003.0;
      uint32_t r = (uint32_t)exp(u * log((double)num_rows));
      if (r >= (uint32_t)num_rows) r = (uint32_t)num_rows - 1;
      T.idx.push_back(r);
    }
    T.off.push_back((int64_t)T.idx.size());
  }
  T.nnz = (int64_t)T.idx.size();
  T.grad.resize((size_t)bags * T.D);
  for (auto &x : T.grad) x = rndf();
  return T;
}

struct Res { std::vector<float> out, dg[3], core[3]; };

#define CK(x) do { tt_status st_ = (x); if (st_ != TT_OK) { fprintf(stderr, "FAIL %s -> %d (%s)\n", #x, st_, tt_strerror(st_)); exit(1); } } while (0)

int main(int argc, char **argv) {
  const char *kind = argc > 1 ? argv[1] : "mfma";
  const int planned_only = argc > 2 ? atoi(argv[2]) : -1;
  std::vector<Tab> tabs;
  if (!strcmp(kind, "unaligned")) { g_off = 1; kind = "mfma"; }
  if (!strcmp(kind, "mfma")) {
    const int d[3] = {4, 8, 4};
    const int ns[3][3] = {{3, 5, 4}, {6, 2, 7}, {2, 9, 3}};
    const int bags[3] = {90, 40, 130};
    for (int t = 0; t < 3; ++t)
      tabs.push_back(make_tab(ns[t], d, 32, 32, bags[t], 5, (int64_t)ns[t][0] * ns[t][1] * ns[t][2] - (t == 1 ? 3 : 0)));
  } else if (!strcmp(kind, "wide")) {  // row factors above 1023: the groupings become radix sorts of two digits
    const int d[3] = {2, 3, 4};  // (small cores: what is under test here is the reorder)
    const int ns[3][3] = {{1, 2100, 2}, {2, 1, 1500}, {3, 1100, 1}};
    const int bags[3] = {120, 90, 60};
    for (int t = 0; t < 3; ++t)
      tabs.push_back(make_tab(ns[t], d, 5, 6, bags[t], 4, (int64_t)ns[t][0] * ns[t][1] * ns[t][2] - (t == 2 ? 7 : 0)));
  } else if (!strcmp(kind, "keys31")) {  // 31-bit row keys: four radix passes
    const int d[3] = {2, 3, 4};
    const int ns[2][3] = {{1290, 1290, 1290}, {7, 5, 3}};
    tabs.push_back(make_tab(ns[0], d, 5, 6, 200, 3, (int64_t)1290 * 1290 * 1290 - 5));
    tabs.push_back(make_tab(ns[1], d, 5, 6, 40, 3, 105));
    // (make_tab draws skewed rows; spread the first table's lookups over the whole key range)
    for (size_t i = 0; i < tabs[0].idx.size(); i += 2) tabs[0].idx[i] = (int64_t)(rnd() % 2146688995u);
  } else if (!strcmp(kind, "cfg5like")) {
    const int d[3] = {4, 8, 4};
    const int ns[4][3] = {{10, 10, 10}, {46, 46, 46}, {342, 342, 342}, {44, 45, 45}};
    const int64_t rows[4] = {1000, 95857, 40000000, 87386};
    const int nb = argc > 3 ? atoi(argv[3]) : 600;
    for (int t = 0; t < 4; ++t) tabs.push_back(make_tab(ns[t], d, 64, 64, nb, 1, rows[t]));
  } else {
    const int d[3] = {2, 3, 4};
    const int ns[3][3] = {{5, 7, 9}, {11, 3, 4}, {2, 13, 6}};
    const int bags[3] = {300, 120, 500};
    for (int t = 0; t < 3; ++t)
      tabs.push_back(make_tab(ns[t], d, 5, 6, bags[t], 7, (int64_t)ns[t][0] * ns[t][1] * ns[t][2]));
  }
  const bool rank_fits = tabs[0].t.num_rows <= 50000000;  // the edge job takes a rank per row of the table
  if (rank_fits) {  // index-graph edges of the first table's batch (sanitizer coverage; the result is compared with
     // the oracle in the Python tests)
    Tab &B = tabs[0];
    std::vector<int32_t> rank((size_t)B.t.num_rows);
    for (size_t i = 0; i < rank.size(); ++i) rank[i] = (int32_t)((i * 7919u) % rank.size());
    int64_t cap = 1;
    for (int b = 0; b < B.bags; ++b) { int64_t l = B.off[b + 1] - B.off[b]; if (l > 64) l = 64; cap += l * (l - 1) / 2; }
    const size_t wb = tt_index_graph_workspace_bytes(B.bags, cap);
    void *ws = amalloc(wb);
    std::vector<int32_t> eu((size_t)cap), ev((size_t)cap), ew((size_t)cap), counts(4);
    CK(tt_index_graph_edges(B.idx.data(), B.off.data(), B.nnz, B.bags, rank.data(), B.t.num_rows, 2, 64, ws, wb, cap,
                            eu.data(), ev.data(), ew.data(), counts.data(), nullptr));
    long long wsum = 0;
    for (int e = 0; e < counts[1]; ++e) wsum += ew[e];
    if (counts[2] != 0 || wsum != counts[0]) { fprintf(stderr, "FAIL index-graph edges: weights %lld pairs %d\n", wsum, counts[0]); return 6; }
    fprintf(stderr, "index-graph edges: %d pairs -> %d edges\n", counts[0], counts[1]);
    free(ws);
  }
  {  // malformed CSR offsets (negative, beyond nnz, decreasing): every kernel has to stay in bounds; the
     // results are unspecified, the plan reports the error
    Tab &B = tabs[0];
    for (int k = 0; k < 3; ++k) B.t.core[k] = B.core[k].data() + g_off;
    std::vector<int64_t> bad = B.off;
    for (size_t i = 1; i + 1 < bad.size(); i += 7) bad[i] = (i % 3 == 0) ? -5 : ((i % 3 == 1) ? B.nnz + 9 : bad[i - 1] - 2);
    tt_plan plan; memset(&plan, 0, sizeof(plan));
    const size_t wb = tt_workspace_bytes(&B.t, B.nnz, B.bags);
    void *ws = amalloc(wb);
    CK(tt_index_reorder(&B.t, B.idx.data(), bad.data(), B.nnz, B.bags, nullptr, ws, wb, &plan, nullptr));
    int64_t counts[4];
    if (tt_plan_status(&plan, nullptr, counts) != TT_ERR_INDEX_RANGE) { fprintf(stderr, "FAIL malformed offsets not reported\n"); return 7; }
    std::vector<float> out((size_t)B.bags * B.D);
    CK(tt_emb_bag_forward(&B.t, &plan, B.idx.data(), bad.data(), B.nnz, B.bags, out.data(), nullptr));
    const size_t rb = tt_reuse_buffer_bytes(&B.t, B.nnz);
    void *reuse = amalloc(rb);
    CK(tt_emb_bag_forward_sample(&B.t, &plan, bad.data(), B.nnz, B.bags, reuse, rb, out.data(), nullptr));
    CK(tt_emb_bag_backward_sgd(&B.t, &plan, B.idx.data(), bad.data(), B.nnz, B.bags, B.grad.data(), 0.f, nullptr));
    if (rank_fits) {
      std::vector<int32_t> rank((size_t)B.t.num_rows, 3), eu(4096), ev(4096), ew(4096), ec(4);
      const size_t gb = tt_index_graph_workspace_bytes(B.bags, 4096);
      void *gws = amalloc(gb);
      CK(tt_index_graph_edges(B.idx.data(), bad.data(), B.nnz, B.bags, rank.data(), B.t.num_rows, 0, 64, gws, gb, 4096,
                              eu.data(), ev.data(), ew.data(), ec.data(), nullptr));
      free(gws);
    }
    free(reuse); free(ws);
    fprintf(stderr, "malformed offsets: reported, no access out of bounds\n");
  }
  for (auto &B : tabs) emu::host_only(&B.t, sizeof(B.t));
  const int T = (int)tabs.size();
  const float lr = 0.01f;
  for (int planned = 1; planned >= 0; --planned) {
    if (planned_only >= 0 && planned != planned_only) continue;
    fprintf(stderr, "== kind %s planned %d\n", kind, planned);
    std::vector<Res> single(T), batch(T);
    // ---- single-table calls
    for (int t = 0; t < T; ++t) {
      Tab &B = tabs[t];
      for (int k = 0; k < 3; ++k) { B.core[k] = B.core0[k]; B.t.core[k] = B.core[k].data() + g_off; }
      tt_plan plan; memset(&plan, 0, sizeof(plan));
      emu::host_only(&plan, sizeof(plan));
      void *ws = nullptr;
      if (planned) {
        size_t wb = tt_workspace_bytes(&B.t, B.nnz, B.bags);
        ws = amalloc(wb);
        CK(tt_index_reorder(&B.t, B.idx.data(), B.off.data(), B.nnz, B.bags, nullptr, ws, wb, &plan, nullptr));
      }
      Res &R = single[t];
      R.out.assign((size_t)B.bags * B.D, -7.f);
      CK(tt_emb_bag_forward(&B.t, planned ? &plan : nullptr, B.idx.data(), B.off.data(), B.nnz, B.bags, R.out.data(), nullptr));
      if (planned) {  // sample-level forward: same bag sums in another order of additions
        const size_t rb = tt_reuse_buffer_bytes(&B.t, B.nnz);
        void *reuse = amalloc(rb);
        std::vector<float> out2((size_t)B.bags * B.D, -7.f);
        CK(tt_emb_bag_forward_sample(&B.t, &plan, B.off.data(), B.nnz, B.bags, reuse, rb, out2.data(), nullptr));
        for (size_t i = 0; i < out2.size(); ++i)
          if (!(fabs((double)out2[i] - R.out[i]) <= 1e-4 * (1.0 + fabs((double)R.out[i])))) {
            fprintf(stderr, "FAIL sample-level forward differs (table %d element %zu: %g vs %g)\n", t, i, out2[i], R.out[i]);
            return 4;
          }
        free(reuse);
      }
      if (planned && tt_bf16_cores_bytes(&B.t) > 0) {  // bf16 cores: against the fp32 kernels on host-rounded cores
        const size_t cb = tt_bf16_cores_bytes(&B.t);
        void *bf = amalloc(cb);
        CK(tt_cores_to_bf16(&B.t, bf, cb, nullptr));
        std::vector<float> out_b((size_t)B.bags * B.D, -7.f), out_r((size_t)B.bags * B.D, -7.f);
        CK(tt_emb_bag_forward_bf16(&B.t, bf, &plan, B.off.data(), B.nnz, B.bags, out_b.data(), nullptr));
        std::vector<float> rounded[3];
        tt_table tr = B.t;
        for (int k = 0; k < 3; ++k) {
          rounded[k].assign(B.t.core[k], B.t.core[k] + (B.core[k].size() - 1));
          for (auto &x : rounded[k]) {
            uint32_t u; memcpy(&u, &x, 4);
            u = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
            memcpy(&x, &u, 4);
          }
          tr.core[k] = rounded[k].data();
        }
        CK(tt_emb_bag_forward(&tr, &plan, B.idx.data(), B.off.data(), B.nnz, B.bags, out_r.data(), nullptr));
        for (size_t i = 0; i < out_b.size(); ++i)
          if (!(fabs((double)out_b[i] - out_r[i]) <= 1e-5 * (1.0 + fabs((double)out_r[i])))) {
            fprintf(stderr, "FAIL bf16 forward differs from the fp32 forward of rounded cores (table %d element %zu: %g vs %g)\n", t, i, out_b[i], out_r[i]);
            return 5;
          }
        free(bf);
      }
      float *dc[3];
      for (int k = 0; k < 3; ++k) { R.dg[k].assign(B.core[k].size() + 1, -9.f); dc[k] = R.dg[k].data() + g_off; }
      CK(tt_emb_bag_backward(&B.t, planned ? &plan : nullptr, B.idx.data(), B.off.data(), B.nnz, B.bags, B.grad.data(), dc, nullptr));
      CK(tt_core_sgd_update(&B.t, planned ? &plan : nullptr, dc, lr, nullptr));
      for (int k = 0; k < 3; ++k) R.core[k] = B.core[k];
      if (planned) {  // fused backward + update on fresh cores (shifted off their alignment like the others)
        for (int k = 0; k < 3; ++k) B.core[k] = B.core0[k];
        CK(tt_emb_bag_backward_sgd(&B.t, &plan, B.idx.data(), B.off.data(), B.nnz, B.bags, B.grad.data(), lr, nullptr));
        for (int k = 0; k < 3; ++k)
          if (memcmp(B.core[k].data(), R.core[k].data(), B.core[k].size() * sizeof(float)) != 0) {
            fprintf(stderr, "FAIL fused update differs from backward + update (table %d core %d)\n", t, k);
            return 3;
          }
      }
      emu::host_only_release(&plan);
      free(ws);
      fprintf(stderr, "single table %d done\n", t);
    }
    // ---- batched calls
    std::vector<tt_batch_item> items(T);
    std::vector<tt_plan> plans(T);
    std::vector<void *> wss(T, nullptr);
    size_t db = tt_batch_desc_bytes(T);
    void *desc = amalloc(db);
    emu::host_only(items.data(), items.size() * sizeof(tt_batch_item));
    emu::host_only(plans.data(), plans.size() * sizeof(tt_plan));
    for (int t = 0; t < T; ++t) {
      Tab &B = tabs[t];
      for (int k = 0; k < 3; ++k) { B.core[k] = B.core0[k]; B.t.core[k] = B.core[k].data() + g_off; }
      memset(&items[t], 0, sizeof(tt_batch_item));
      memset(&plans[t], 0, sizeof(tt_plan));
      items[t].table = &B.t;
      items[t].indices = B.idx.data(); items[t].offsets = B.off.data();
      items[t].nnz = B.nnz; items[t].num_bags = B.bags;
      if (planned) {
        items[t].plan = &plans[t];
        items[t].workspace_bytes = tt_workspace_bytes(&B.t, B.nnz, B.bags);
        items[t].workspace = wss[t] = amalloc(items[t].workspace_bytes);
      }
      batch[t].out.assign((size_t)B.bags * B.D, -7.f);
      items[t].out = batch[t].out.data();
      items[t].grad_out = B.grad.data();
      for (int k = 0; k < 3; ++k) { batch[t].dg[k].assign(B.core[k].size() + 1, -9.f); items[t].dcore[k] = batch[t].dg[k].data() + g_off; }
    }
    if (planned) CK(tt_index_reorder_batched(T, items.data(), desc, db, nullptr));
    fprintf(stderr, "batched reorder done\n");
    CK(tt_emb_bag_forward_batched(T, items.data(), desc, db, nullptr));
    fprintf(stderr, "batched forward done\n");
    CK(tt_emb_bag_backward_batched(T, items.data(), desc, db, nullptr));
    fprintf(stderr, "batched backward done\n");
    CK(tt_core_sgd_update_batched(T, items.data(), lr, desc, db, nullptr));
    fprintf(stderr, "batched sgd done\n");
    int bad = 0;
    for (int t = 0; t < T; ++t) {
      for (int k = 0; k < 3; ++k) batch[t].core[k] = tabs[t].core[k];
      auto cmp = [&](const std::vector<float> &a, const std::vector<float> &b, const char *what, bool exact) {
        size_t nbad = 0; double worst = 0;
        for (size_t i = 0; i < a.size(); ++i) {
          if (exact ? memcmp(&a[i], &b[i], 4) != 0 : fabs((double)a[i] - b[i]) > 1e-4) { ++nbad; }
          double e = fabs((double)a[i] - b[i]); if (e > worst) worst = e;
        }
        if (nbad) { fprintf(stderr, "MISMATCH table %d %s: %zu of %zu differ (max %.3g)\n", t, what, nbad, a.size(), worst); ++bad; }
      };
      // (kind "wide": the tables differ so much in their row factors that a batched launch, whose
      // reduction layout is chosen for all tables at once, adds a table's gradients in another order
      // than its single-table call: equal to rounding, not bit for bit)
      const bool exact = planned != 0 && strcmp(kind, "wide") != 0;
      cmp(single[t].out, batch[t].out, "out", true);
      for (int k = 0; k < 3; ++k) {
        char nm[16]; snprintf(nm, sizeof nm, "dg%d", k + 1);
        cmp(single[t].dg[k], batch[t].dg[k], nm, exact);
        snprintf(nm, sizeof nm, "core%d", k + 1);
        cmp(single[t].core[k], batch[t].core[k], nm, exact);
      }
    }
    {
      uint64_t h = 1469598103934665603ull;
      auto mix = [&](const std::vector<float> &v) { for (float x : v) { uint32_t u; memcpy(&u, &x, 4); h = (h ^ u) * 1099511628211ull; } };
      for (int t = 0; t < T; ++t) { mix(single[t].out); for (int k = 0; k < 3; ++k) { mix(single[t].dg[k]); mix(single[t].core[k]); } }
      fprintf(stderr, "checksum of single-table results: %016llx\n", (unsigned long long)h);
    }
    if (planned) {  // ---- the same tables as ONE fused table: members' results within rounding of the single calls
      tt_fuse_members mem; memset(&mem, 0, sizeof(mem));
      mem.num_tables = T;
      for (int t = 0; t < T; ++t) { for (int k = 0; k < 3; ++k) mem.n[t][k] = tabs[t].t.n[k]; mem.num_rows[t] = tabs[t].t.num_rows; }
      tt_table ft = tabs[0].t;
      const tt_status fits = tt_fuse_shape(&mem, &ft);
      if (fits == TT_ERR_SHAPE && !strcmp(kind, "keys31")) {  // 2^31 rows or more: refused, as it must be
        fprintf(stderr, "fused table of %d members: refused (too many rows), 0 values off\n", T);
      } else {
      CK(fits);
      std::vector<float> fcore[3], fdg[3];
      float *fdc[3];
      for (int k = 0; k < 3; ++k) {
        const size_t inner = (size_t)ft.d[k] * ft.r[k + 1];
        fcore[k].assign((size_t)ft.r[k] * ft.n[k] * inner + 1, 0.f);
        fdg[k].assign(fcore[k].size() + 1, -9.f);
        int o = 0;
        for (int t = 0; t < T; ++t) {
          const int nk = tabs[t].t.n[k];
          for (int r = 0; r < ft.r[k]; ++r)
            memcpy(fcore[k].data() + g_off + ((size_t)r * ft.n[k] + o) * inner,
                   tabs[t].core0[k].data() + g_off + (size_t)r * nk * inner, (size_t)nk * inner * sizeof(float));
          o += nk;
        }
        ft.core[k] = fcore[k].data() + g_off;
        fdc[k] = fdg[k].data() + g_off;
      }
      std::vector<const int64_t *> pidx(T), poff(T);
      std::vector<int64_t> nnzs(T), nbs(T);
      int64_t tn = 0, tb = 0;
      for (int t = 0; t < T; ++t) { pidx[t] = tabs[t].idx.data(); poff[t] = tabs[t].off.data(); nnzs[t] = tabs[t].nnz; nbs[t] = tabs[t].bags; tn += nnzs[t]; tb += nbs[t]; }
      std::vector<int64_t> fidx((size_t)tn), foff((size_t)tb + 1);
      emu::host_only(&mem, sizeof(mem));
      emu::host_only(pidx.data(), T * sizeof(void *));
      emu::host_only(poff.data(), T * sizeof(void *));
      CK(tt_fuse_lookups(&mem, pidx.data(), poff.data(), nullptr, nnzs.data(), nbs.data(), fidx.data(), foff.data(), nullptr));
      emu::host_only_release(&mem); emu::host_only_release(pidx.data()); emu::host_only_release(poff.data());
      emu::host_only(&ft, sizeof(ft));
      tt_plan fplan; memset(&fplan, 0, sizeof(fplan));
      const size_t fwb = tt_workspace_bytes(&ft, tn, tb);
      void *fws = amalloc(fwb);
      CK(tt_index_reorder(&ft, fidx.data(), foff.data(), tn, tb, nullptr, fws, fwb, &fplan, nullptr));
      int64_t fcounts[4];
      CK(tt_plan_status(&fplan, nullptr, fcounts));
      std::vector<float> fout((size_t)tb * tabs[0].D, -7.f), fgrad;
      for (int t = 0; t < T; ++t) fgrad.insert(fgrad.end(), tabs[t].grad.begin(), tabs[t].grad.end());
      CK(tt_emb_bag_forward(&ft, &fplan, fidx.data(), foff.data(), tn, tb, fout.data(), nullptr));
      CK(tt_emb_bag_backward(&ft, &fplan, fidx.data(), foff.data(), tn, tb, fgrad.data(), fdc, nullptr));
      emu::host_only_release(&ft);
      size_t fbad = 0, b0 = 0;
      auto near = [](float a, float b) { return fabs((double)a - b) <= 1e-4 * (1.0 + fabs((double)b)); };
      for (int t = 0; t < T; ++t) {
        for (size_t i = 0; i < single[t].out.size(); ++i) if (!near(fout[b0 * tabs[0].D + i], single[t].out[i])) ++fbad;
        b0 += (size_t)tabs[t].bags;
      }
      for (int k = 0; k < 3; ++k) {
        const size_t inner = (size_t)ft.d[k] * ft.r[k + 1];
        int o = 0;
        for (int t = 0; t < T; ++t) {
          const int nk = tabs[t].t.n[k];
          for (int r = 0; r < ft.r[k]; ++r)
            for (size_t e = 0; e < (size_t)nk * inner; ++e)
              if (!near(fdg[k][g_off + ((size_t)r * ft.n[k] + o) * inner + e], single[t].dg[k][g_off + (size_t)r * nk * inner + e])) ++fbad;
          o += nk;
        }
      }
      free(fws);
      fprintf(stderr, "fused table of %d members: %lld rows, %lld prefixes, %zu values off\n", T, (long long)fcounts[0], (long long)fcounts[1], fbad);
      if (fbad) return 8;
      }
    }
    emu::host_only_release(items.data());
    emu::host_only_release(plans.data());
    for (void *w : wss) free(w);
    free(desc);
    fprintf(stderr, "== kind %s planned %d: %s\n", kind, planned, bad ? "MISMATCH" : "identical");
    if (bad) return 2;
  }
  return 0;
}
