// SparseAttn for bf16 storage, d = 128, 64-token blocks: the dense-contraction part of the
// path, on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, float32 accumulation).
//
// Work split.  One wavefront owns one query block (64 queries) and walks that block's own
// list of kept key blocks; there is no cross-wave communication and no workgroup barrier.  A
// workgroup is four such wavefronts (four consecutive query blocks), one per SIMD, each with
// a private 32 KB LDS region (K tile 64x128 and transposed V tile 128x64).
//
// Per key tile a wave computes
//     S^T = K Q^T      (keys x queries, 2x2 MFMA tiles of 32x32, 8 k-steps over d)
//     online softmax over keys
//     O^T += V^T P^T   (d x queries, 4x2 MFMA tiles, 4 k-steps over the 64 keys)
// The transposed forms put the query on the lane axis of every accumulator (lane l holds
// query l%32 of a 32-query group), so the row statistics of the softmax are per-lane
// scalars: the max / sum over keys run down a lane's own registers plus one exchange
// between lanes l and l^32, and rescaling O is one multiply per register.
//
// Operand feeding.  A 32x32x16 MFMA takes, per lane, 8 consecutive contraction elements of
// one row.  K rows (d contiguous) and V^T rows (keys contiguous; V arrives block-transposed
// from the reorder step) give those as single 16-byte LDS reads; Q lives in registers for
// the whole list; P is built in registers.  Lane l feeds K row sigma(l%32) where sigma swaps
// bits 2 and 3: with that choice the 8 scores a lane holds in accumulator registers
// 8t..8t+7 belong to keys 16t + 8*(l/32) + 0..7, exactly the 8 contraction elements the
// P^T operand of the second product needs, so P goes from accumulator to operand with no
// cross-lane movement.
//
// Memory.  K/V tiles travel HBM/L2 -> LDS with 16-byte direct-to-LDS loads (no registers
// in between); each lane fetches the chunk that belongs at its LDS position, and the
// position is XOR-swizzled with the row so that the 16-byte operand reads are free of bank
// conflicts.  The K load of tile j+1 is issued right after S of tile j, the V load after
// the second product, so each has a softmax + a product to land.
#include <math.h>
#include <stdlib.h>
#include "da_internal.h"

namespace da {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;
constexpr int BS = 64;
constexpr int K_TILE = BS * D * 2;   // 16 KB, rows of 256 B
constexpr int V_TILE = D * BS * 2;   // 16 KB, rows of 128 B
constexpr int WAVE_LDS = K_TILE + V_TILE;
constexpr int O_STRIDE = D * 2 + 16; // padded row stride of the output staging area

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* gbl_ptr;

// 16 KB tile, rows of ROWB bytes, moved 1 KB (64 lanes x 16 B) per step: the lane at LDS
// position p of row r fetches global chunk p ^ swizzle(r).  `src` and `lds` are wave-uniform;
// the per-lane part of the address is a 32-bit offset (`loff[it & 3]` + a constant), so the
// loads take the scalar-base + vector-offset form.
template <int ROWB>
__device__ inline void tile_lane_offsets(int lane, unsigned loff[4]) {
  constexpr int CPR = ROWB / 16;        // chunks per row
  constexpr int RPS = 64 / CPR;         // rows per step
  const int r_in = lane / CPR, p = lane % CPR;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    int row = a * RPS + r_in;           // the swizzle of row it*RPS + r_in only depends on it & 3
    int sw = ROWB == 256 ? (row & 15) : ((row >> 1) & 7);
    loff[a] = r_in * ROWB + ((p ^ sw) << 4);
  }
}

template <bool DIRECT, int ROWB>
__device__ inline void load_tile(const unsigned char* __restrict__ src, unsigned char* lds, int lane,
                                 const unsigned loff[4]) {
  constexpr int RPS = 64 / (ROWB / 16);
#pragma unroll
  for (int it = 0; it < 16; ++it) {
    const unsigned char* g = src + it * RPS * ROWB + loff[it & 3];
    if (DIRECT) {
      __builtin_amdgcn_global_load_lds((gbl_ptr)g, (lds_ptr)(lds + it * 1024), 16, 0, 0);
    } else {
      *(uint4*)(lds + it * 1024 + lane * 16) = *(const uint4*)g;
    }
  }
}

__device__ inline int sigma(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

template <bool DIRECT>
__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(Geo q, const unsigned char* __restrict__ Qp,
                                                          const unsigned char* __restrict__ Kp,
                                                          const unsigned char* __restrict__ Vt,
                                                          const int32_t* __restrict__ idx, unsigned char* __restrict__ Op,
                                                          float* __restrict__ lse, int wg_per_xcd, long long total_qb) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * WAVE_LDS];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, lives in SGPRs
  const int lane = threadIdx.x & 63;
  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous range of
  // query blocks so that neighbouring blocks (similar key lists) share that XCD's L2.
  const int xcd = blockIdx.x & 7;
  const long long lwg = (long long)xcd * wg_per_xcd + (blockIdx.x >> 3);
  const long long qb = lwg * 4 + wave;           // over (batch*head, block)
  if (qb >= total_qb) return;                    // whole wave leaves; no barrier is used below
  const long long bh = qb / q.g;
  unsigned char* kl = smem + wave * WAVE_LDS;
  unsigned char* vl = kl + K_TILE;
  const unsigned char* Kbh = Kp + bh * q.n_pad * (D * 2);
  const unsigned char* Vbh = Vt + bh * q.n_pad * (D * 2);
  const int32_t* list = idx + qb * q.k;
  const int per_frame = q.gh * q.gw;

  const int r = lane & 31, hh = lane >> 5;
  unsigned koff[4], voff[4];
  tile_lane_offsets<256>(lane, koff);
  tile_lane_offsets<128>(lane, voff);

  // Q fragments: B operand, lane (query r of group nt, half hh) holds d = 16t + 8hh .. +7
  bf16x8 qf[2][8];
  {
    const unsigned char* qbase = Qp + (qb * BS) * (D * 2);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int t = 0; t < 8; ++t)
        qf[nt][t] = *(const bf16x8*)(qbase + (32 * nt + r) * (D * 2) + (16 * t + 8 * hh) * 2);
  }

  // per-lane LDS read offsets
  const int krow = sigma(r);
  const int ke = (hh ^ (krow & 15)) << 4;        // swizzled chunk offset, XORed with 32*t below
  const int ve = (hh ^ ((r >> 1) & 7)) << 4;

  f32x16 o[4][2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][nt][i] = 0.f;
  float m[2] = {-INFINITY, -INFINITY};
  float l[2] = {0.f, 0.f};
  const float c2 = 0.08838834764831845f * 1.4426950408889634f;   // log2(e)/sqrt(128)

  int j = __builtin_amdgcn_readfirstlane(list[0]);
  load_tile<DIRECT, 256>(Kbh + (long long)j * K_TILE, kl, lane, koff);
  load_tile<DIRECT, 128>(Vbh + (long long)j * V_TILE, vl, lane, voff);

  for (int t_list = 0; t_list < q.k; ++t_list) {
    const int jn = __builtin_amdgcn_readfirstlane(list[min(t_list + 1, q.k - 1)]);
    // valid slots of key block j (pad slots sit at the tail of a block)
    int nv;
    {
      int rr = j % per_frame;
      int bi = rr / q.gw, bj = rr - bi * q.gw;
      nv = min(q.ph, q.fh - bi * q.ph) * min(q.pw, q.fw - bj * q.pw);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // ---- S^T = K Q^T
    f32x16 s[2][2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[mt][nt][i] = 0.f;
    {
      bf16x8 ka[16];                             // all 16 K operands are requested up front
#pragma unroll
      for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
          ka[2 * t + mt] = *(const bf16x8*)(kl + (32 * mt + krow) * 256 + ((32 * t) ^ ke));
#pragma unroll
      for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          s[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[2 * t + mt], qf[0][t], s[mt][0], 0, 0, 0);
          s[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[2 * t + mt], qf[1][t], s[mt][1], 0, 0, 0);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (t_list + 1 < q.k) load_tile<DIRECT, 256>(Kbh + (long long)jn * K_TILE, kl, lane, koff);

    // ---- pad keys out of the softmax: accumulator register i of tile mt is key
    //      32*mt + 16*(i>>3) + 8*hh + (i&7)
    if (nv < BS) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int key = 32 * mt + 16 * (i >> 3) + 8 * hh + (i & 7);
          if (key >= nv) {
            s[mt][0][i] = -INFINITY;
            s[mt][1][i] = -INFINITY;
          }
        }
    }

    // ---- online softmax, per query = per lane
    bf16x8 pf[2][4];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      float mx = s[0][nt][0];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[mt][nt][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m[nt], mx);     // finite: slot 0 of every block is valid
      const float alpha = __builtin_amdgcn_exp2f((m[nt] - m_new) * c2);
      m[nt] = m_new;
      const float mc = m_new * c2;
      float lsum = 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mt][nt][i], c2, -mc));
          float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mt][nt][i + 1], c2, -mc));
          lsum += p0 + p1;
          f32x2 pp = {p0, p1};
          bf16x2 pb = __builtin_convertvector(pp, bf16x2);
          pf[nt][2 * mt + (i >> 3)][i & 7] = pb[0];
          pf[nt][2 * mt + (i >> 3)][(i & 7) + 1] = pb[1];
        }
      l[nt] = l[nt] * alpha + lsum;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][nt][i] *= alpha;
    }

    // ---- O^T += V^T P^T
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    {
      bf16x8 va[16];
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
          va[4 * t + dt] = *(const bf16x8*)(vl + (32 * dt + r) * 128 + ((32 * t) ^ ve));
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          o[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[4 * t + dt], pf[0][t], o[dt][0], 0, 0, 0);
          o[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[4 * t + dt], pf[1][t], o[dt][1], 0, 0, 0);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (t_list + 1 < q.k) load_tile<DIRECT, 128>(Vbh + (long long)jn * V_TILE, vl, lane, voff);
    j = jn;
  }

  // ---- epilogue: normalise, convert, stage through LDS, write rows of 256 B
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float lt = l[nt] + __shfl_xor(l[nt], 32);
    const float inv = 1.0f / lt;
    if (lse && hh == 0) lse[qb * BS + 32 * nt + r] = m[nt] * 0.08838834764831845f + __logf(lt);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        // registers 4a..4a+3 are d = 32dt + 8a + 4hh + 0..3 of query 32nt + r
        f32x2 v0 = {o[dt][nt][4 * a] * inv, o[dt][nt][4 * a + 1] * inv};
        f32x2 v1 = {o[dt][nt][4 * a + 2] * inv, o[dt][nt][4 * a + 3] * inv};
        bf16x2 b0 = __builtin_convertvector(v0, bf16x2);
        bf16x2 b1 = __builtin_convertvector(v1, bf16x2);
        uint2 w = make_uint2(*(unsigned*)&b0, *(unsigned*)&b1);
        *(uint2*)(kl + (32 * nt + r) * O_STRIDE + (32 * dt + 8 * a + 4 * hh) * 2) = w;
      }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  unsigned char* obase = Op + (qb * BS) * (D * 2);
#pragma unroll
  for (int it = 0; it < 16; ++it) {
    int row = it * 4 + (lane >> 4), ch = lane & 15;
    *(uint4*)(obase + row * (D * 2) + ch * 16) = *(const uint4*)(kl + row * O_STRIDE + ch * 16);
  }
}

hipError_t launch_attn_bf16(const Geo& q, const void* Qp, const void* Kp, const void* Vt, const int32_t* idx, void* Op,
                            float* lse, hipStream_t s) {
  long long total_qb = (long long)q.B * q.H * q.g;
  long long wgs = (total_qb + 3) / 4;
  int wg_per_xcd = (int)((wgs + 7) / 8);
  unsigned grid = (unsigned)(wg_per_xcd * 8);
  // DA_ATTN_STAGED=1 selects the variant that stages tiles through registers instead of
  // direct-to-LDS loads (same LDS image, same results); a debugging aid.
  const char* env = getenv("DA_ATTN_STAGED");
  if (env && env[0] == '1')
    hipLaunchKernelGGL(attn_bf16_kernel<false>, dim3(grid), dim3(256), 0, s, q, (const unsigned char*)Qp,
                       (const unsigned char*)Kp, (const unsigned char*)Vt, idx, (unsigned char*)Op, lse, wg_per_xcd,
                       total_qb);
  else
    hipLaunchKernelGGL(attn_bf16_kernel<true>, dim3(grid), dim3(256), 0, s, q, (const unsigned char*)Qp,
                       (const unsigned char*)Kp, (const unsigned char*)Vt, idx, (unsigned char*)Op, lse, wg_per_xcd,
                       total_qb);
  return hipGetLastError();
}

}  // namespace da
