// Average pooling of Q and K inside each latent frame (Definition 3.2); with MAXP the maximum instead
// (the other downsampling kernel of the ablation, Section 4.3).
// HBM-bound: Q and K are read once in 16-byte pieces straight from the original layout
// (the tokens of a patch row are contiguous); each lane owns a fixed group of channels of
// one block and adds the block's tokens in slot order, so the float32 result does not
// depend on the launch shape:  acc = acc + x (one rounding per add), mean = acc / valid.
// Q and K are read once and never again by this pass: the loads are marked non-temporal, so the stream does not
// push anything else out of the L2 (measured on the headline shape: 5.4 -> 5.8 TB/s).
#include "da_internal.h"

#pragma clang fp contract(off)

namespace da {

// 16 bytes, read once
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 load_once(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <int DT>
struct Vec;
template <>
struct Vec<DA_BF16> {
  static constexpr int N = 8;
  __device__ static void widen(const uint4& r, float* f) {
    const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f[2 * j] = __uint_as_float(w[j] << 16);
      f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
  }
};
template <>
struct Vec<DA_F32> {
  static constexpr int N = 4;
  __device__ static void widen(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

constexpr int kPoolThreads = 64;

// grid.x covers (bh, block, chunk) items; grid.y = 0 for Q, 1 for K.  With REORDER the tokens are
// also written, as they go by, to their slots of the reordered tensors Qp, Kp (Algorithm 1), pad
// slots zeroed: pooling and reordering then read Q and K once between them.
template <int DT, bool REORDER, bool MAXP>
__global__ __launch_bounds__(kPoolThreads) void pool_kernel(Geo q, const uint4* __restrict__ Q, const uint4* __restrict__ K,
                                                   float* __restrict__ q_pool, float* __restrict__ k_pool,
                                                   uint4* __restrict__ Qp, uint4* __restrict__ Kp, int cpr,
                                                   long long items) {
  constexpr int N = Vec<DT>::N;
  long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (item >= items) return;
  const uint4* X = blockIdx.y ? K : Q;
  float* out = blockIdx.y ? k_pool : q_pool;
  long long blk = item / cpr;  // over bh * g
  int c = (int)(item - blk * cpr);
  long long bh = blk / q.g;
  int i = (int)(blk - bh * q.g);
  BlockPos b = block_pos(q, i);
  // chunks between consecutive rows of the source, rows between the block's patch rows
  const long long sn = q.in.sn / N;
  const long long pitch = block_row_pitch(q, b);
  const uint4* src = X + row_offset(q.in, q.H, bh, block_first_row(q, i, b)) / N + c;
  uint4* const dbase = blockIdx.y ? Kp : Qp;          // NULL: this tensor is only pooled
  const bool wr = REORDER && dbase != nullptr;
  uint4* dstp = wr ? dbase + (blk * q.block) * cpr + c : nullptr;   // slot 0 of the block
  float acc[N];
#pragma unroll
  for (int j = 0; j < N; ++j) acc[j] = MAXP ? -INFINITY : 0.f;
  // one token's channels go into the running sum, or (MAXP) replace the running maximum where larger
  auto take = [&](const float (&f)[N]) {
#pragma unroll
    for (int j = 0; j < N; ++j) acc[j] = MAXP ? (f[j] > acc[j] ? f[j] : acc[j]) : acc[j] + f[j];
  };
  int u = 0;
  // two full patch rows at a time where the patch is 8 wide: sixteen independent loads in flight,
  // added in slot order
  if (b.vw == 8) {
    for (; u + 2 <= b.vh; u += 2) {
      const uint4* row = src + (long long)u * pitch * sn;
      uint4 r[16];
#pragma unroll
      for (int t = 0; t < 16; ++t) r[t] = load_once(&row[((long long)(t >> 3) * pitch + (t & 7)) * sn]);
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        if (wr) dstp[(long long)(u * 8 + t) * cpr] = r[t];
        float f[N];
        Vec<DT>::widen(r[t], f);
        take(f);
      }
    }
  }
  for (; u < b.vh; ++u) {
    const uint4* row = src + (long long)u * pitch * sn;
    int v = 0;
    for (; v + 8 <= b.vw; v += 8) {  // eight independent loads in flight, added in order
      uint4 r[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) r[t] = load_once(&row[(long long)(v + t) * sn]);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        if (wr) dstp[(long long)(u * b.vw + v + t) * cpr] = r[t];
        float f[N];
        Vec<DT>::widen(r[t], f);
        take(f);
      }
    }
    for (; v < b.vw; ++v) {
      const uint4 rv = load_once(&row[(long long)v * sn]);
      if (wr) dstp[(long long)(u * b.vw + v) * cpr] = rv;
      float f[N];
      Vec<DT>::widen(rv, f);
      take(f);
    }
  }
  if (wr)
    for (int sl = b.vh * b.vw; sl < q.block; ++sl) dstp[(long long)sl * cpr] = make_uint4(0u, 0u, 0u, 0u);
  float cnt = (float)(b.vh * b.vw);
  float* dst = out + blk * q.d + c * N;
#pragma unroll
  for (int j = 0; j < N; ++j) dst[j] = MAXP ? acc[j] : acc[j] / cnt;   // IEEE division (correctly rounded is the compiler default for HIP)
}

hipError_t launch_pool(const Geo& q, const void* Q, const void* K, float* q_pool, float* k_pool, hipStream_t s) {
  return launch_pool_reorder(q, Q, K, q_pool, k_pool, nullptr, nullptr, s);
}

// Qp, Kp: each may be NULL (that tensor is then only pooled)
hipError_t launch_pool_reorder(const Geo& q, const void* Q, const void* K, float* q_pool, float* k_pool, void* Qp,
                               void* Kp, hipStream_t s) {
  size_t es = q.dtype == DA_BF16 ? 2 : 4;
  int cpr = (int)(q.d * es / 16);
  long long items = (long long)q.B * q.H * q.g * cpr;
  dim3 grid((unsigned)((items + kPoolThreads - 1) / kPoolThreads), 2);
  const bool re = Qp != nullptr || Kp != nullptr;
  const bool mx = q.pool == DA_POOL_MAX;
#define DA_POOL_LAUNCH(DT, RE, MX)                                                                                    \
  hipLaunchKernelGGL((pool_kernel<DT, RE, MX>), grid, dim3(kPoolThreads), 0, s, q, (const uint4*)Q, (const uint4*)K,  \
                     q_pool, k_pool, (uint4*)Qp, (uint4*)Kp, cpr, items)
#define DA_POOL_PICK(DT)                                          \
  if (re && mx) DA_POOL_LAUNCH(DT, true, true);                   \
  else if (re) DA_POOL_LAUNCH(DT, true, false);                   \
  else if (mx) DA_POOL_LAUNCH(DT, false, true);                   \
  else DA_POOL_LAUNCH(DT, false, false)
  if (q.dtype == DA_BF16) {
    DA_POOL_PICK(DA_BF16);
  } else {
    DA_POOL_PICK(DA_F32);
  }
#undef DA_POOL_PICK
#undef DA_POOL_LAUNCH
  return hipGetLastError();
}

}  // namespace da
