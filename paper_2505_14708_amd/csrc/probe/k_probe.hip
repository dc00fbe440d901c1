// Measuring sticks (da_probe.h): a pure matrix-instruction loop and a plain copy.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "da.h"
#include "da_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeGrid = 256 * 4;     // four workgroups of eight waves per CU's worth
constexpr int kProbeThreads = 512;

__global__ __launch_bounds__(512, 2) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
  // operands: pseudo-random finite values in [-1, 1), different per lane and register
  bf16x8 a[4], b[4];
  unsigned x = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      x = x * 1664525u + 1013904223u;
      a[i][j] = (__bf16)((float)(int)(x >> 8) * (1.0f / 8388608.0f) - 1.0f);
      x = x * 1664525u + 1013904223u;
      b[i][j] = (__bf16)((float)(int)(x >> 8) * (1.0f / 8388608.0f) - 1.0f);
    }
  f32x16 c[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) c[i][j] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(t + i) & 3], b[t], c[i], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(a[i]));   // keep the loop a loop
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += c[i][j];
  sink[(blockIdx.x * 512u + threadIdx.x) & ((1u << 20) - 1u)] = s;
}

// 16 bytes that are read once / written once and not needed in the caches afterwards
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ inline u32x4 load_once(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ inline void store_once(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// a plain copy: a workgroup of 512 takes 64 KB in a row per trip (eight 16-byte loads in flight per lane, then eight
// stores), workgroups stride over the buffer
__global__ __launch_bounds__(512) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  constexpr size_t kPer = 512 * 8;
  size_t base = (size_t)blockIdx.x * kPer;
  for (; base + kPer <= n16; base += (size_t)gridDim.x * kPer) {
    u32x4 r[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) r[t] = load_once(src + base + t * 512 + threadIdx.x);
#pragma unroll
    for (int t = 0; t < 8; ++t) store_once(dst + base + t * 512 + threadIdx.x, r[t]);
  }
  if (base < n16)
    for (size_t i = base + threadIdx.x; i < n16; i += 512) dst[i] = src[i];
}

// a plain read: a workgroup of 512 takes 128 KB in a row per trip (sixteen 16-byte loads in flight per lane, each
// load of a wave one contiguous KB), workgroups stride over the buffer; what was read is folded into one word per lane
__global__ __launch_bounds__(512) void probe_read_kernel(const uint4* __restrict__ src, unsigned* __restrict__ sink, size_t n16) {
  constexpr size_t kPer = 512 * 16;
  unsigned acc = 0u;
  size_t base = (size_t)blockIdx.x * kPer;
  for (; base + kPer <= n16; base += (size_t)gridDim.x * kPer) {
    uint4 r[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) r[t] = src[base + t * 512 + threadIdx.x];
#pragma unroll
    for (int t = 0; t < 16; ++t) acc ^= r[t].x ^ r[t].y ^ r[t].z ^ r[t].w;
  }
  if (base < n16)                                       // the last, partial stretch
    for (size_t i = base + threadIdx.x; i < n16; i += 512) {
      const uint4 r = src[i];
      acc ^= r.x ^ r.y ^ r.z ^ r.w;
    }
  sink[(blockIdx.x * 512u + threadIdx.x) & ((1u << 20) - 1u)] = acc;
}

}  // namespace

extern "C" {

int da_probe_mfma_bf16(int iters, float* sink, double* flop, void* stream) {
  if (!sink || !flop) return DA_ERR_NULL;
  if (iters < 1) return DA_ERR_DIM;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeGrid), dim3(kProbeThreads), 0, (hipStream_t)stream, sink, iters);
  *flop = (double)kProbeGrid * (kProbeThreads / 64) * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}

int da_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return DA_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return DA_ERR_DIM;
  if (((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return DA_ERR_ALIGN;
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 64), dim3(512), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst,
                     bytes / 16);
  return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}

int da_probe_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink) return DA_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return DA_ERR_DIM;
  if ((uintptr_t)src & 15u) return DA_ERR_ALIGN;
  hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 64), dim3(512), 0, (hipStream_t)stream, (const uint4*)src, (unsigned*)sink,
                     bytes / 16);
  return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}

}  // extern "C"
