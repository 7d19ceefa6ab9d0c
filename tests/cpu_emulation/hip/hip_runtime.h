// CPU stand-in for the parts of the HIP runtime and device language the TT kernels use.
// One workgroup runs at a time on a pool of OS threads (one per lane), so that
// AddressSanitizer / UBSan see every memory access of a kernel.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#include <functional>

struct dim3 {
  unsigned x, y, z;
  dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct alignas(8) float2 { float x, y; };
struct alignas(16) float4 { float x, y, z, w; };
static inline float4 make_float4(float x, float y, float z, float w) { return float4{x, y, z, w}; }
struct alignas(16) int4 { int x, y, z, w; };
struct alignas(8) int2 { int x, y; };
static inline int4 make_int4(int x, int y, int z, int w) { return int4{x, y, z, w}; }
struct alignas(16) uint4 { unsigned x, y, z, w; };
struct alignas(8) uint2 { unsigned x, y; };
static inline uint2 make_uint2(unsigned x, unsigned y) { return uint2{x, y}; }
static inline float __uint_as_float(unsigned u) { float f; memcpy(&f, &u, 4); return f; }
static inline unsigned __float_as_uint(float f) { unsigned u; memcpy(&u, &f, 4); return u; }

typedef void *hipStream_t;
typedef void *hipEvent_t;
typedef int hipError_t;
enum { hipSuccess = 0 };
enum { hipMemcpyDeviceToHost = 2, hipMemcpyHostToDevice = 1 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };

namespace emu {
extern thread_local dim3 t_threadIdx;
extern dim3 g_blockIdx, g_blockDim, g_gridDim;
void launch(dim3 grid, dim3 block, size_t lds, const char *name, const std::function<void()> &body);
void host_only(const void *p, size_t n);   // a region kernels must not touch: poisoned (ASan) while a launch runs
void host_only_release(const void *p);
void syncthreads();
void *dyn_lds();
uint64_t wave_exchange(uint64_t v, int src_lane);          // value of lane src_lane (own lane if out of range)
uint64_t wave_ballot(bool pred);
void wave_mfma_16x16x4(float a, float b, float *c4);
}  // namespace emu

#define threadIdx emu::t_threadIdx
#define blockIdx emu::g_blockIdx
#define blockDim emu::g_blockDim
#define gridDim emu::g_gridDim

#define __global__
#define __device__
#define __host__
#define __shared__ static
#define __align__(n) __attribute__((aligned(n)))
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)

#define hipLaunchKernelGGL(kernel, grid, block, lds, stream, ...) \
  emu::launch(grid, block, lds, #kernel, [=]() { kernel(__VA_ARGS__); })

#define hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, start_event, stop_event, flags, ...) \
  emu::launch(grid, block, lds, #kernel, [=]() { kernel(__VA_ARGS__); })

static inline hipError_t hipGetLastError() { return hipSuccess; }
static inline hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
enum { hipDeviceAttributeMultiprocessorCount = 1 };
static inline hipError_t hipDeviceGetAttribute(int *v, int, int) { *v = 4; return hipSuccess; }  // few "compute units": the work queues are exercised
#define HIP_SYMBOL(x) (&(x))
static inline hipError_t hipGetSymbolAddress(void **p, const void *symbol) { *p = const_cast<void *>(symbol); return hipSuccess; }
static inline hipError_t hipFuncSetAttribute(const void *, int, int) { return hipSuccess; }
static inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, int, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
static inline hipError_t hipEventCreate(hipEvent_t *e) { *e = nullptr; return hipSuccess; }
static inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
static inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }

static inline void __syncthreads() { emu::syncthreads(); }
static inline int __lane() { return (int)(emu::t_threadIdx.x & 63); }
static inline int __shfl_up(int v, int delta, int = 64) {
  return (int)(uint32_t)emu::wave_exchange((uint32_t)v, __lane() - delta);
}
static inline int __shfl(int v, int src, int width = 64) {  // src counts inside the lane's segment of `width` lanes
  return (int)(uint32_t)emu::wave_exchange((uint32_t)v, (__lane() & ~(width - 1)) | (src & (width - 1)));
}
static inline int __ffsll(unsigned long long v) { return __builtin_ffsll((long long)v); }
static inline float __shfl_xor(float v, int mask, int = 64) {
  uint32_t u; memcpy(&u, &v, 4);
  u = (uint32_t)emu::wave_exchange(u, __lane() ^ mask);
  float r; memcpy(&r, &u, 4); return r;
}
static inline unsigned long long __ballot(bool p) { return emu::wave_ballot(p); }
static inline int __popcll(unsigned long long v) { return __builtin_popcountll(v); }
static inline int __builtin_amdgcn_readfirstlane(int v) { return (int)(uint32_t)emu::wave_exchange((uint32_t)v, -2); }
static inline int __builtin_amdgcn_readlane(int v, int lane) { return (int)(uint32_t)emu::wave_exchange((uint32_t)v, lane); }
// lanes are fibers that run one after the other between collectives: a point that orders LDS
// accesses inside a wavefront has to be one
static inline void __builtin_amdgcn_wave_barrier() { emu::wave_exchange(0, -1); }
#define __builtin_amdgcn_fence(order, scope) ((void)0)
static inline long long clock64() { return 0; }

static inline int atomicAdd(int *p, int v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
static inline void __threadfence() { __atomic_thread_fence(__ATOMIC_SEQ_CST); }
static inline int atomicOr(int *p, int v) { return __atomic_fetch_or(p, v, __ATOMIC_RELAXED); }
static inline float atomicAdd(float *p, float v) {
  uint32_t *u = reinterpret_cast<uint32_t *>(p);
  uint32_t old = __atomic_load_n(u, __ATOMIC_RELAXED);
  for (;;) {
    float f; memcpy(&f, &old, 4);
    f += v;
    uint32_t nu; memcpy(&nu, &f, 4);
    if (__atomic_compare_exchange_n(u, &old, nu, false, __ATOMIC_RELAXED, __ATOMIC_RELAXED)) { memcpy(&f, &old, 4); return f; }
  }
}

typedef float emu_f32x4 __attribute__((ext_vector_type(4)));
static inline emu_f32x4 emu_mfma(float a, float b, emu_f32x4 c, int, int, int) {
  float t[4] = {c[0], c[1], c[2], c[3]};
  emu::wave_mfma_16x16x4(a, b, t);
  return (emu_f32x4){t[0], t[1], t[2], t[3]};
}
#define __builtin_amdgcn_mfma_f32_16x16x4f32 emu_mfma
// 16x16x16 bf16: lane l supplies A[m = l%16][k = 4*(l/16) + i] and B[k = 4*(l/16) + i][n = l%16],
// i = 0..3 -- the sum over i of four 16x16x4 products of the widened values
typedef short emu_bf16x4 __attribute__((ext_vector_type(4)));
static inline emu_f32x4 emu_mfma_bf16(emu_bf16x4 a, emu_bf16x4 b, emu_f32x4 c, int, int, int) {
  float t[4] = {c[0], c[1], c[2], c[3]};
  for (int i = 0; i < 4; ++i)
    emu::wave_mfma_16x16x4(__uint_as_float((unsigned)(unsigned short)a[i] << 16),
                           __uint_as_float((unsigned)(unsigned short)b[i] << 16), t);
  return (emu_f32x4){t[0], t[1], t[2], t[3]};
}
#define __builtin_amdgcn_mfma_f32_16x16x16bf16_1k emu_mfma_bf16
