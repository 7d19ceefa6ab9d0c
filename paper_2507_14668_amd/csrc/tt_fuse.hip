// Fused tables: the lookups of several TT tables that share column factors and ranks are mapped
// into one TT table whose cores are the members' cores side by side along the row-factor axis
// (block-diagonal index space).  A member's row keeps its three slices (index split of Section
// III-B, applied per member, then shifted by the member's ranges), so every kernel of the path runs
// unchanged on the fused table -- with one launch where the members would take one each.
#include "tt_internal.h"

namespace {

struct FuseMember {
  int n2, n3;             // row factors 2 and 3 of the member (factor 1 follows from the quotient)
  int o1, o2, o3;         // the member's first index in every fused core
  int pad;
  long long num_rows;     // valid rows of the member
  long long l0, b0;       // first fused lookup / first fused bag of the member
  long long nnz, bags;
  const int64_t *idx, *off, *remap;
};
struct FuseArgs {
  int T, N2, N3, pad;
  long long total_nnz, total_bags;
  FuseMember m[TT_FUSE_MAX_TABLES];
};
static_assert(sizeof(FuseArgs) <= 3600, "the members travel as kernel arguments");

// grid (tiles, members): thread p of member t maps lookup p and offset p of that member
__global__ void __launch_bounds__(TT_BLOCK)
k_fuse_lookups(FuseArgs a, int64_t *__restrict__ fused_idx, int64_t *__restrict__ fused_off) {
  const FuseMember &m = a.m[blockIdx.y];
  const long long span = m.nnz > m.bags ? m.nnz : m.bags;
  for (long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x; p < span;
       p += (long long)gridDim.x * blockDim.x) {
    if (p < m.nnz) {
      long long i = m.idx[p];
      if (m.remap && i >= 0 && i < m.num_rows) i = m.remap[i];
      long long v = -1;
      if (i >= 0 && i < m.num_rows) {
        const long long pre = i / m.n3, i3 = i - pre * m.n3, i1 = pre / m.n2, i2 = pre - i1 * m.n2;
        v = ((m.o1 + i1) * a.N2 + m.o2 + i2) * a.N3 + m.o3 + i3;
      }
      fused_idx[m.l0 + p] = v;
    }
    if (p < m.bags) {  // offset p of the member; its last one (== nnz) is the next member's first
      const long long o = m.off[p];
      bool ok = o >= 0 && o <= m.nnz && (p != 0 || o == 0);
      if (p == m.bags - 1) ok = ok && m.off[m.bags] == m.nnz;
      fused_off[m.b0 + p] = ok ? m.l0 + o : -1;
    }
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) fused_off[a.total_bags] = a.total_nnz;
}

}  // namespace

tt_status ttk_fuse_shape(const tt_fuse_members *mem, long long N[3]) {
  if (!mem || mem->num_tables < 1 || mem->num_tables > TT_FUSE_MAX_TABLES) return TT_ERR_INVALID_ARG;
  N[0] = N[1] = N[2] = 0;
  for (int t = 0; t < mem->num_tables; ++t) {
    long long cap = 1;
    for (int k = 0; k < 3; ++k) {
      if (mem->n[t][k] < 1) return TT_ERR_SHAPE;
      N[k] += mem->n[t][k];
      cap *= mem->n[t][k];
    }
    if (mem->num_rows[t] < 1 || mem->num_rows[t] > cap) return TT_ERR_SHAPE;
  }
  // the same limits a table has: 31-bit row keys and prefix ids
  if (N[0] >= 2147483647LL || N[1] >= 2147483647LL || N[2] >= 2147483647LL) return TT_ERR_SHAPE;
  if (N[0] * N[1] >= 2147483647LL || N[0] * N[1] * N[2] >= 2147483647LL) return TT_ERR_SHAPE;
  return TT_OK;
}

tt_status ttk_fuse_lookups(const tt_fuse_members *mem, const int64_t *const *indices,
                           const int64_t *const *offsets, const int64_t *const *remaps,
                           const int64_t *nnz, const int64_t *num_bags, int64_t *fused_indices,
                           int64_t *fused_offsets, hipStream_t s) {
  long long N[3];
  tt_status st = ttk_fuse_shape(mem, N);
  if (st != TT_OK) return st;
  if (!indices || !offsets || !nnz || !num_bags || !fused_offsets) return TT_ERR_INVALID_ARG;
  FuseArgs a = {};
  a.T = mem->num_tables; a.N2 = (int)N[1]; a.N3 = (int)N[2];
  long long o[3] = {0, 0, 0}, l0 = 0, b0 = 0, span = 1;
  for (int t = 0; t < a.T; ++t) {
    if (nnz[t] < 0 || num_bags[t] < 0 || (num_bags[t] == 0 && nnz[t] != 0)) return TT_ERR_INVALID_ARG;
    if (!offsets[t] || (nnz[t] > 0 && !indices[t])) return TT_ERR_INVALID_ARG;
    FuseMember &m = a.m[t];
    m.n2 = mem->n[t][1]; m.n3 = mem->n[t][2];
    m.o1 = (int)o[0]; m.o2 = (int)o[1]; m.o3 = (int)o[2];
    m.num_rows = mem->num_rows[t];
    m.l0 = l0; m.b0 = b0; m.nnz = nnz[t]; m.bags = num_bags[t];
    m.idx = indices[t]; m.off = offsets[t]; m.remap = remaps ? remaps[t] : nullptr;
    for (int k = 0; k < 3; ++k) o[k] += mem->n[t][k];
    l0 += nnz[t]; b0 += num_bags[t];
    const long long sp = nnz[t] > num_bags[t] ? nnz[t] : num_bags[t];
    if (sp > span) span = sp;
  }
  if (l0 >= 2147483647LL || b0 >= 2147483647LL) return TT_ERR_INVALID_ARG;
  if (l0 > 0 && !fused_indices) return TT_ERR_INVALID_ARG;
  a.total_nnz = l0; a.total_bags = b0;
  long long tiles = tt_ceil_div(span, TT_BLOCK);
  if (tiles > 4096) tiles = 4096;
  hipLaunchKernelGGL(k_fuse_lookups, dim3((unsigned)tiles, (unsigned)a.T), dim3(TT_BLOCK), 0, s, a,
                     fused_indices, fused_offsets);
  return tt_launch_status();
}
