// Draft logits L = Q~ K~^T / sqrt(d) and the draft attention map softmax(L) (Definition 3.2).
//
// The kept-block decision is taken from these logits, so they are evaluated in float32 with
// one fixed order that a CPU can repeat bit for bit: acc = fma(q[c], k[c], acc) for c ascending
// (the IEEE fused multiply-add: one instruction and one rounding per term; no matrix cores, no
// split sums), then one multiply by float(1/sqrt(d)).  The work is a register-tiled product
// on the vector ALUs: a workgroup owns a 128x128 tile of L, a thread an 8x8 piece; Q~ and K~
// pieces go through LDS transposed so a thread reads its 8 rows / 8 columns as 16-byte loads.
#include <math.h>
#include "da_internal.h"

// The compiler contracts nothing in this file (the pragma covers the code below, and the build also
// passes -ffp-contract=off for it): the only fused multiply-adds are the ones written out.
#pragma clang fp contract(off)

namespace da {

constexpr int TM = 128;   // tile rows (query blocks) and columns (key blocks)
constexpr int TC = 16;    // channels per LDS stage

__global__ __launch_bounds__(256) void draft_logits_kernel(Geo q, const float* __restrict__ q_pool,
                                                           const float* __restrict__ k_pool, float* __restrict__ logits,
                                                           float scale) {
  __shared__ __attribute__((aligned(16))) float qs[TC][TM];
  __shared__ __attribute__((aligned(16))) float ks[TC][TM];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const long long bh = blockIdx.z;
  const int row0 = blockIdx.y * TM, col0 = blockIdx.x * TM;
  const float* qb = q_pool + bh * (long long)q.g * q.d;
  const float* kb = k_pool + bh * (long long)q.g * q.d;
  float acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = 0.f;

  // loader: thread -> (row r = tid/2, half of the TC channels), as 16-byte loads (d is a multiple of 4).  The next
  // stage's loads are asked for before the current stage is multiplied.
  const int lr = tid >> 1, lc = (tid & 1) * (TC / 2);
  const int gr = row0 + lr, gc = col0 + lr;
  const float* qrow = qb + (long long)min(gr, q.g - 1) * q.d;
  const float* krow = kb + (long long)min(gc, q.g - 1) * q.d;
  float4 nq[2], nk[2];
  auto fetch = [&](int c0) {
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int c = c0 + lc + 4 * v;
      const bool in = c < q.d;                          // (a group of four is inside the row or outside it as a whole)
      nq[v] = in && gr < q.g ? *(const float4*)(qrow + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      nk[v] = in && gc < q.g ? *(const float4*)(krow + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  fetch(0);
  for (int c0 = 0; c0 < q.d; c0 += TC) {
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      qs[lc + 4 * v + 0][lr] = nq[v].x; qs[lc + 4 * v + 1][lr] = nq[v].y;
      qs[lc + 4 * v + 2][lr] = nq[v].z; qs[lc + 4 * v + 3][lr] = nq[v].w;
      ks[lc + 4 * v + 0][lr] = nk[v].x; ks[lc + 4 * v + 1][lr] = nk[v].y;
      ks[lc + 4 * v + 2][lr] = nk[v].z; ks[lc + 4 * v + 3][lr] = nk[v].w;
    }
    __syncthreads();
    if (c0 + TC < q.d) fetch(c0 + TC);
    const int cend = min(TC, q.d - c0);
    for (int c = 0; c < cend; ++c) {
      float a[8], b[8];
      // rows ty*4..+3 and 64+ty*4..+3; columns tx*4..+3 and 64+tx*4..+3
      *(float4*)&a[0] = *(const float4*)&qs[c][ty * 4];
      *(float4*)&a[4] = *(const float4*)&qs[c][64 + ty * 4];
      *(float4*)&b[0] = *(const float4*)&ks[c][tx * 4];
      *(float4*)&b[4] = *(const float4*)&ks[c][64 + tx * 4];
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* out = logits + bh * (long long)q.g * q.g;
  // a thread's columns come in two runs of four: with g a multiple of 4 a run is inside the row or outside it as a
  // whole, and 16-byte aligned, so it goes out as one store
  const bool vec = (q.g & 3) == 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int r = row0 + (i < 4 ? ty * 4 + i : 64 + ty * 4 + (i - 4));
    if (r >= q.g) continue;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = col0 + 64 * h + tx * 4;
      float* dst = out + (long long)r * q.g + c;
      if (vec) {
        if (c < q.g)
          *(float4*)dst = make_float4(acc[i][4 * h] * scale, acc[i][4 * h + 1] * scale, acc[i][4 * h + 2] * scale,
                                      acc[i][4 * h + 3] * scale);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (c + j < q.g) dst[j] = acc[i][4 * h + j] * scale;
      }
    }
  }
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One wavefront per row; safe in place (every element is read before it is written by the
// same lane, and rows do not overlap).
__global__ __launch_bounds__(256) void row_softmax_kernel(const float* logits, float* draft, int g, long long rows) {
  long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  int lane = threadIdx.x & 63;
  const float* in = logits + row * g;
  float* out = draft + row * g;
  float m = -INFINITY;
  for (int j = lane; j < g; j += 64) m = fmaxf(m, in[j]);
  m = wave_max(m);
  float z = 0.f;
  for (int j = lane; j < g; j += 64) z += expf(in[j] - m);
  z = wave_sum(z);
  float inv = 1.0f / z;
  for (int j = lane; j < g; j += 64) out[j] = expf(in[j] - m) * inv;
}

hipError_t launch_draft_logits(const Geo& q, const float* q_pool, const float* k_pool, float* logits, hipStream_t s) {
  unsigned t = (unsigned)((q.g + TM - 1) / TM);
  float scale = (float)(1.0 / sqrt((double)q.d));
  dim3 grid(t, t, (unsigned)(q.B * q.H));
  hipLaunchKernelGGL(draft_logits_kernel, grid, dim3(256), 0, s, q, q_pool, k_pool, logits, scale);
  return hipGetLastError();
}

hipError_t launch_row_softmax(const Geo& q, const float* logits, float* draft, hipStream_t s) {
  long long rows = (long long)q.B * q.H * q.g;
  hipLaunchKernelGGL(row_softmax_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, logits, draft, q.g, rows);
  return hipGetLastError();
}

}  // namespace da
