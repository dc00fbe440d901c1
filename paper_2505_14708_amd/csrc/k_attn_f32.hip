// SparseAttn for float32 storage: float32 arithmetic throughout on the vector ALUs (no
// down-conversion for the matrix cores), so the small float32 configuration can be checked
// to 1e-4.  It is a correctness path, not a fast one.
//
// One wavefront per query block of 64 slots; lane u owns query slot u (its q row, its output
// row, its running max and sum).  For each kept key block the K tile [64][D] and the
// transposed V tile [D][64] are staged in LDS; all lanes read the same K row / V column at
// the same time (LDS broadcast).
#include <math.h>
#include "da_internal.h"

namespace da {

template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(Geo q, const float* __restrict__ Qp, const float* __restrict__ Kp,
                                                      const float* __restrict__ Vt, const int32_t* __restrict__ idx,
                                                      const int32_t* __restrict__ row_ptr, long long cap,
                                                      float* __restrict__ Op, float* __restrict__ lse) {
  extern __shared__ __attribute__((aligned(16))) float smem_f[];
  float* ks = smem_f;            // [64][D]
  float* vs = smem_f + 64 * D;   // [D][64]
  const int lane = threadIdx.x;
  const long long qb = blockIdx.x;          // over bh * g
  const long long bh = qb / q.g;
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const float* qrow = Qp + (qb * 64 + lane) * D;
  float qv[D], o[D];
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    float4 t = *(const float4*)(qrow + c);
    qv[c] = t.x; qv[c + 1] = t.y; qv[c + 2] = t.z; qv[c + 3] = t.w;
  }
#pragma unroll
  for (int c = 0; c < D; ++c) o[c] = 0.f;
  float m = -INFINITY, l = 0.f;
  // k columns per row, or (row_ptr given) lists of any length, one after the other per head
  const int32_t* list = idx + qb * q.k;
  int len = q.k;
  if (row_ptr) {
    const int32_t* rp = row_ptr + bh * (q.g + 1) + (qb - bh * q.g);
    // (offsets that are not what the interface asks for are brought into the head's stretch, and an entry that is no
    // block number is left out: such lists give unspecified results, but nothing outside the arrays is touched)
    const int begin = min(max(rp[0], 0), (int)cap);
    list = idx + bh * cap + begin;
    len = min(max(rp[1] - begin, 0), (int)cap - begin);
  }
  for (int t = 0; t < len; ++t) {
    int j = list[t];
    if ((unsigned)j >= (unsigned)q.g) continue;          // (the same in every lane)
    int nv = block_valid(q, j);
    const float4* ksrc = (const float4*)(Kp + (bh * q.n_pad + (long long)j * 64) * D);
    const float4* vsrc = (const float4*)(Vt + (bh * q.g + j) * (long long)D * 64);
    __syncthreads();
    for (int e = lane; e < 64 * D / 4; e += 64) {
      ((float4*)ks)[e] = ksrc[e];
      ((float4*)vs)[e] = vsrc[e];
    }
    __syncthreads();
    for (int v0 = 0; v0 < 64; v0 += 8) {       // eight keys at a time
      float s[8];
      float grp_max = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) acc = fmaf(qv[c], ks[(v0 + e) * D + c], acc);
        acc = (v0 + e) < nv ? acc : -INFINITY;  // pad keys are never attended
        s[e] = acc;
        grp_max = fmaxf(grp_max, acc);
      }
      // slot 0 of every block is valid, so the running max is finite from the first group on
      float m_new = fmaxf(m, grp_max);
      float alpha = exp2f((m - m_new) * scale_log2);
      l *= alpha;
#pragma unroll
      for (int c = 0; c < D; ++c) o[c] *= alpha;
      m = m_new;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float p = exp2f((s[e] - m) * scale_log2);
        l += p;
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = fmaf(p, vs[c * 64 + v0 + e], o[c]);
      }
    }
  }
  const float inv = l > 0.f ? 1.0f / l : 0.f;   // an empty list: zero rows
  float* orow = Op + (qb * 64 + lane) * D;
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    float4 t = make_float4(o[c] * inv, o[c + 1] * inv, o[c + 2] * inv, o[c + 3] * inv);
    *(float4*)(orow + c) = t;
  }
  if (lse) lse[qb * 64 + lane] = l > 0.f ? m * (float)(1.0 / sqrt((double)D)) + logf(l) : -INFINITY;
}

hipError_t launch_attn_f32(const Geo& q, const float* Qp, const float* Kp, const float* Vt, const int32_t* idx,
                           const int32_t* row_ptr, long long cap, float* Op, float* lse, hipStream_t s) {
  unsigned blocks = (unsigned)((long long)q.B * q.H * q.g);
  size_t lds = (size_t)2 * 64 * q.d * sizeof(float);
  if (q.d == 64)
    hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(blocks), dim3(64), lds, s, q, Qp, Kp, Vt, idx, row_ptr, cap, Op, lse);
  else
    hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(blocks), dim3(64), lds, s, q, Qp, Kp, Vt, idx, row_ptr, cap, Op, lse);
  return hipGetLastError();
}

}  // namespace da
