// Reduced-precision storage of the TT cores: bf16 copies, fp32 arithmetic (the paper's deployment
// discussion names half-precision-capable devices; the cores are the only stored parameters).
//
// k_cores_to_bf16 rounds the three fp32 cores to bf16 (round to nearest, ties to even) into one
// caller buffer in the layout the bf16 forward kernel reads:
//   core 0  [n1][d1][R1]                       as stored
//   core 1  [n2][R1 / 4][d2 * R2][4]           the four consecutive r1 of one (j2, r2) column adjacent
//   core 2  [R2][n3][d3]                       as stored
// each part starting at a multiple of 256 bytes.
#include "tt_internal.h"

namespace {

__device__ __forceinline__ unsigned short float_to_bf16_rne(float f) {
  const unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // NaN stays NaN
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

__global__ void __launch_bounds__(TT_BLOCK)
k_cores_to_bf16(TTShape sh, const float *__restrict__ g1, const float *__restrict__ g2,
                const float *__restrict__ g3, unsigned short *__restrict__ o1,
                unsigned short *__restrict__ o2, unsigned short *__restrict__ o3) {
  const long long len1 = (long long)sh.n1 * sh.S1, len2 = (long long)sh.R1 * sh.n2 * sh.S2,
                  len3 = (long long)sh.R2 * sh.n3 * sh.d3;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < len1 + len2 + len3; e += stride) {
    if (e < len1) {
      o1[e] = float_to_bf16_rne(g1[e]);
    } else if (e < len1 + len2) {
      // output element ((i2 * R1/4 + r1q) * S2 + col) * 4 + i  <-  G2[r1 = 4*r1q + i][i2][col]
      const long long o = e - len1;
      const int i = (int)(o & 3);
      const long long rest = o >> 2;
      const int col = (int)(rest % sh.S2);
      const long long t = rest / sh.S2;
      const int r1q = (int)(t % (sh.R1 / 4)), i2 = (int)(t / (sh.R1 / 4));
      o2[o] = float_to_bf16_rne(g2[((size_t)(4 * r1q + i) * sh.n2 + i2) * sh.S2 + col]);
    } else {
      o3[e - len1 - len2] = float_to_bf16_rne(g3[e - len1 - len2]);
    }
  }
}

size_t pad256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

void ttk_bf16_layout(const TTShape &sh, size_t off[3], size_t *total) {
  off[0] = 0;
  off[1] = pad256((size_t)sh.n1 * sh.S1 * 2);
  off[2] = off[1] + pad256((size_t)sh.R1 * sh.n2 * sh.S2 * 2);
  *total = off[2] + pad256((size_t)sh.R2 * sh.n3 * sh.d3 * 2);
}

tt_status ttk_cores_to_bf16(const TTShape &sh, const float *const core[3], void *buf, hipStream_t s) {
  size_t off[3], total;
  ttk_bf16_layout(sh, off, &total);
  char *base = (char *)buf;
  const long long elems = (long long)sh.n1 * sh.S1 + (long long)sh.R1 * sh.n2 * sh.S2 + (long long)sh.R2 * sh.n3 * sh.d3;
  long long blocks = (elems + TT_BLOCK - 1) / TT_BLOCK;
  if (blocks > 8192) blocks = 8192;
  const float *c0 = core[0], *c1 = core[1], *c2 = core[2];  // read the host array here, not in the launch expression
  hipLaunchKernelGGL(k_cores_to_bf16, dim3((unsigned)blocks), dim3(TT_BLOCK), 0, s, sh, c0, c1, c2,
                     (unsigned short *)(base + off[0]), (unsigned short *)(base + off[1]),
                     (unsigned short *)(base + off[2]));
  return tt_launch_status();
}
