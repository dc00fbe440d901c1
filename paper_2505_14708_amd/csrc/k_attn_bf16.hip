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
// conflicts.  The loads are issued from inline assembly and waited for with explicit
// s_waitcnt vmcnt(N), so a wait covers exactly the tile that is needed and the younger
// prefetch stays in flight.
//
// Software pipeline (the matrix pipe and the vector ALU of a SIMD run concurrently when the
// instruction stream interleaves independent work):
//     stage 1:  S of tile t+1 on the matrix cores  ||  exp / sum / pack of tile t on the VALU
//     stage 2:  O += V P of tile t on the matrix cores  ||  row max of tile t+1 on the VALU
// with the K load of tile t+2 issued after stage 1 and the V load of tile t+1 after stage 2.
// The running max is only moved (and O rescaled) when a row max exceeds it by more than 2^8
// in the exponent's units; until then probabilities are formed against the stale max, which
// is exact after the final division because numerator and denominator share it.
#include <math.h>
#include <stdlib.h>
#include <string.h>
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
constexpr float kScale = 0.08838834764831845f;               // 1/sqrt(128)
constexpr float kC2 = 0.08838834764831845f * 1.4426950408889634f;   // log2(e)/sqrt(128)
constexpr float kLazy = 8.0f;        // move the running max only past this many powers of two

typedef __attribute__((address_space(3))) unsigned char* lds_bytes;

// ------------------------------------------------------------------------------------------
// tile movement
// ------------------------------------------------------------------------------------------
// 16 KB tile, rows of ROWB bytes, moved 1 KB (64 lanes x 16 B) per step: the lane at LDS
// position p of row r fetches global chunk p ^ swizzle(r).  Step `it` covers rows
// it*RPS .. it*RPS+RPS-1 (RPS*ROWB = 1024), so its global and LDS offsets are both it*1024
// plus a per-lane part that only depends on it & 3.
template <int ROWB>
__device__ inline void tile_lane_offsets(int lane, unsigned loff[4]) {
  constexpr int CPR = ROWB / 16;        // chunks per row
  constexpr int RPS = 64 / CPR;         // rows per step
  const int r_in = lane / CPR, p = lane % CPR;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    int row = a * RPS + r_in;
    int sw = ROWB == 256 ? (row & 15) : ((row >> 1) & 7);
    loff[a] = r_in * ROWB + ((p ^ sw) << 4);
  }
}

// Direct-to-LDS load of 16 bytes per lane: lane i's data lands at m0 + 16*i.
__device__ __forceinline__ void dma16(const unsigned char* g, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}

__device__ __forceinline__ void dma_tile(const unsigned char* src, unsigned lds_addr, const unsigned (&loff)[4]) {
#pragma unroll
  for (int it = 0; it < 16; ++it) dma16(src + it * 1024 + loff[it & 3], lds_addr + it * 1024);
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ inline int sigma(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Multiply an accumulator tile that lives in accumulation registers by a per-lane factor.
// Written against the accumulation registers directly so that the (rare) rescale does not make
// the compiler shuttle O between the two register files on every trip of the tile loop.
__device__ __forceinline__ void scale_acc(f32x16& acc, float a) {
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float x = acc[i], tmp;
    asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                 : "+a"(x), "=&v"(tmp)
                 : "v"(a));
    acc[i] = x;
  }
}
// Tell the register allocator that an accumulator tile is wanted in accumulation registers here
// (no instruction is emitted).
__device__ __forceinline__ void pin_acc(f32x16& acc) { asm volatile("" : "+a"(acc)); }
// wait states around scale_acc: matrix results must have been written before they are read, and
// the rewritten registers must be visible to the next matrix instruction
__device__ __forceinline__ void acc_hazard_before() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }
__device__ __forceinline__ void acc_hazard_after() { asm volatile("s_nop 7" ::: "memory"); }

// ------------------------------------------------------------------------------------------
// per-wave state and the pieces of one tile step
// ------------------------------------------------------------------------------------------
struct Lane {
  int r, hh;
  const unsigned char* kread;   // LDS address of this lane's K row, m-tile 0
  const unsigned char* vread;   // LDS address of this lane's V^T row, d-tile 0
  int ke, ve;                   // swizzled chunk offsets (XORed with 32*t)
};

// K operand u = 2t + mt  (t: k-step over d, mt: 32-key half)
__device__ __forceinline__ bf16x8 k_frag(const Lane& L, int u) {
  const int t = u >> 1, mt = u & 1;
  return *(const bf16x8*)(L.kread + mt * (32 * 256) + ((32 * t) ^ L.ke));
}
// V^T operand u = 4t + dt  (t: k-step over keys, dt: 32-channel group)
__device__ __forceinline__ bf16x8 v_frag(const Lane& L, int u) {
  const int t = u >> 2, dt = u & 3;
  return *(const bf16x8*)(L.vread + dt * (32 * 128) + ((32 * t) ^ L.ve));
}

// pad keys out of the softmax: accumulator register i of tile mt is key 32mt + 16(i>>3) + 8hh + (i&7)
__device__ __forceinline__ void mask_pad_keys(f32x16 (&s)[2][2], int nv, int hh) {
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

__device__ __forceinline__ float max16(const f32x16& a, float m) {
#pragma unroll
  for (int i = 0; i < 16; i += 2) m = fmaxf(fmaxf(a[i], a[i + 1]), m);   // v_max3_f32
  return m;
}

// exp / sum / pack of 16 scores (one accumulator tile) of one query group into two P operands
__device__ __forceinline__ void exp_pack(const f32x16& s, float mc, float& lsum, bf16x8& p_lo, bf16x8& p_hi) {
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], kC2, -mc));
    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 1], kC2, -mc));
    lsum += p0;
    lsum += p1;
    f32x2 pp = {p0, p1};
    bf16x2 pb = __builtin_convertvector(pp, bf16x2);
    if (i < 8) {
      p_lo[i] = pb[0];
      p_lo[i + 1] = pb[1];
    } else {
      p_hi[i - 8] = pb[0];
      p_hi[i - 7] = pb[1];
    }
  }
}

struct Soft {
  float m[2];     // reference max per query group (raw score units); -inf before the first tile
  float l[2];     // this lane's partial sum of probabilities
  float mx[2];    // row max of the tile that is about to be exponentiated
};

// One step of the pipeline.  On entry `sc` holds the raw scores of tile t (row max in st.mx),
// the K tile of t+1 and the V tile of t are in flight (in that order).  On exit `sn` holds
// the scores of tile t+1 (max in st.mx), O has tile t added, and the K tile of t+2 and the V
// tile of t+1 are in flight.
template <bool HAS_NEXT>
__device__ __forceinline__ void tile_step(f32x16 (&sc)[2][2], f32x16 (&sn)[2][2], f32x16 (&o)[4][2],
                                          const bf16x8 (&qf)[2][8], Soft& st, const Lane& L,
                                          const unsigned char* k_next2, bool has_next2, const unsigned char* v_next,
                                          int nv_next, unsigned k_lds, unsigned v_lds, const unsigned (&koff)[4],
                                          const unsigned (&voff)[4]) {
  // ---- rare: move the running max and rescale what has been accumulated against it
  {
    bool need = (st.mx[0] - st.m[0]) * kC2 > kLazy || (st.mx[1] - st.m[1]) * kC2 > kLazy;
    if (__any(need)) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float m_new = fmaxf(st.m[nt], st.mx[nt]);
        const float alpha = __builtin_amdgcn_exp2f((st.m[nt] - m_new) * kC2);   // exp2(-inf) = 0 the first time
        st.m[nt] = m_new;
        st.l[nt] *= alpha;
        acc_hazard_before();
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) scale_acc(o[dt][nt], alpha);
        acc_hazard_after();
      }
    }
  }
  const float mc0 = st.m[0] * kC2, mc1 = st.m[1] * kC2;
  bf16x8 pf[2][4];
  float ls0 = 0.f, ls1 = 0.f;

  // ---- stage 1: S(t+1) on the matrix cores, exp/sum/pack of S(t) on the VALU
  if (HAS_NEXT) {
    wait_vm<16>();                       // K(t+1) landed; the 16 loads of V(t) may still fly
    bf16x8 kf[2][4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) sn[mt][nt][i] = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) kf[0][u] = k_frag(L, u);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (g < 3) {
#pragma unroll
        for (int u = 0; u < 4; ++u) kf[(g + 1) & 1][u] = k_frag(L, 4 * (g + 1) + u);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int uu = 4 * g + u, t = uu >> 1, mt = uu & 1;
        sn[mt][0] = mfma(kf[g & 1][u], qf[0][t], sn[mt][0]);
        sn[mt][1] = mfma(kf[g & 1][u], qf[1][t], sn[mt][1]);
      }
      // VALU share of this group: one accumulator tile of S(t)
      if (g == 0) exp_pack(sc[0][0], mc0, ls0, pf[0][0], pf[0][1]);
      if (g == 1) exp_pack(sc[1][0], mc0, ls0, pf[0][2], pf[0][3]);
      if (g == 2) exp_pack(sc[0][1], mc1, ls1, pf[1][0], pf[1][1]);
      if (g == 3) exp_pack(sc[1][1], mc1, ls1, pf[1][2], pf[1][3]);
    }
    wait_lds();                          // every K operand is in registers: the K buffer is free
    if (has_next2) dma_tile(k_next2, k_lds, koff);
  } else {
    exp_pack(sc[0][0], mc0, ls0, pf[0][0], pf[0][1]);
    exp_pack(sc[1][0], mc0, ls0, pf[0][2], pf[0][3]);
    exp_pack(sc[0][1], mc1, ls1, pf[1][0], pf[1][1]);
    exp_pack(sc[1][1], mc1, ls1, pf[1][2], pf[1][3]);
  }
  st.l[0] += ls0;
  st.l[1] += ls1;

  // ---- stage 2: O += V P of tile t on the matrix cores, pad mask + row max of S(t+1) on the VALU
  if (HAS_NEXT && has_next2) wait_vm<16>(); else wait_vm<0>();   // V(t) landed
  if (HAS_NEXT && nv_next < BS) mask_pad_keys(sn, nv_next, L.hh);
  {
    bf16x8 vf[2][4];
    float mx0 = -INFINITY, mx1 = -INFINITY;
#pragma unroll
    for (int u = 0; u < 4; ++u) vf[0][u] = v_frag(L, u);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (g < 3) {
#pragma unroll
        for (int u = 0; u < 4; ++u) vf[(g + 1) & 1][u] = v_frag(L, 4 * (g + 1) + u);
      }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        o[dt][0] = mfma(vf[g & 1][dt], pf[0][g], o[dt][0]);
        o[dt][1] = mfma(vf[g & 1][dt], pf[1][g], o[dt][1]);
      }
      if (HAS_NEXT) {
        if (g == 0) mx0 = max16(sn[0][0], mx0);
        if (g == 1) mx0 = max16(sn[1][0], mx0);
        if (g == 2) mx1 = max16(sn[0][1], mx1);
        if (g == 3) mx1 = max16(sn[1][1], mx1);
      }
    }
    if (HAS_NEXT) {
      st.mx[0] = fmaxf(mx0, __shfl_xor(mx0, 32));
      st.mx[1] = fmaxf(mx1, __shfl_xor(mx1, 32));
    }
    wait_lds();                          // every V operand is in registers: the V buffer is free
    if (HAS_NEXT) dma_tile(v_next, v_lds, voff);
  }
}

__device__ __forceinline__ int valid_slots(const Geo& q, int per_frame, int j) {
  int rr = j % per_frame;
  int bi = rr / q.gw, bj = rr - bi * q.gw;
  return min(q.ph, q.fh - bi * q.ph) * min(q.pw, q.fw - bj * q.pw);
}

__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(Geo q, const unsigned char* __restrict__ Qp,
                                                          const unsigned char* __restrict__ Kp,
                                                          const unsigned char* __restrict__ Vt,
                                                          const int32_t* __restrict__ idx, unsigned char* __restrict__ Op,
                                                          float* __restrict__ lse, int wg_per_xcd, long long total_qb, int map_mode) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * WAVE_LDS];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, lives in SGPRs
  const int lane = threadIdx.x & 63;
  long long qb;                                  // over (batch*head, block)
  if (map_mode == 0) {
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous range of
    // query blocks.
    const int xcd = blockIdx.x & 7;
    const long long lwg = (long long)xcd * wg_per_xcd + (blockIdx.x >> 3);
    qb = lwg * 4 + wave;
    if (qb >= total_qb) return;                  // whole wave leaves; no barrier is used below
  } else {
    // Heads one after the other (so the K/V of the heads in flight fit the last-level cache);
    // inside a head a workgroup is one patch position and four consecutive frames (their key
    // lists overlap most), and the frame groups of one position follow each other on one XCD.
    const int per_frame = q.gh * q.gw;
    const int fgs = (q.T + 3) >> 2;
    const int pos_per_xcd = (per_frame + 7) >> 3;
    const int wg_per_head = 8 * pos_per_xcd * fgs;
    const long long head = blockIdx.x / wg_per_head;
    const int n = blockIdx.x - (int)(head * wg_per_head);
    const int xcd = n & 7, slot = n >> 3;
    const int pos = xcd + 8 * (slot / fgs);
    const int f = 4 * (slot % fgs) + wave;
    if (pos >= per_frame || f >= q.T) return;
    qb = head * q.g + (long long)f * per_frame + pos;
  }
  const long long bh = qb / q.g;
  unsigned char* kl = smem + wave * WAVE_LDS;
  unsigned char* vl = kl + K_TILE;
  const unsigned k_lds = (unsigned)(uintptr_t)(lds_bytes)kl;
  const unsigned v_lds = k_lds + K_TILE;
  const unsigned char* Kbh = Kp + bh * q.n_pad * (D * 2);
  const unsigned char* Vbh = Vt + bh * q.n_pad * (D * 2);
  const int32_t* list = idx + qb * q.k;
  const int per_frame = q.gh * q.gw;
  const int k = q.k;

  Lane L;
  L.r = lane & 31;
  L.hh = lane >> 5;
  const int krow = sigma(L.r);
  L.kread = kl + krow * 256;
  L.vread = vl + L.r * 128;
  L.ke = (L.hh ^ (krow & 15)) << 4;
  L.ve = (L.hh ^ ((L.r >> 1) & 7)) << 4;
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
        qf[nt][t] = *(const bf16x8*)(qbase + (32 * nt + L.r) * (D * 2) + (16 * t + 8 * L.hh) * 2);
  }

  f32x16 o[4][2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][nt][i] = 0.f;
  Soft st;
  st.m[0] = st.m[1] = -INFINITY;
  st.l[0] = st.l[1] = 0.f;

  // ---- prologue: S of the first tile
  f32x16 sa[2][2], sb[2][2];
  int j0 = __builtin_amdgcn_readfirstlane(list[0]);
  int j1 = __builtin_amdgcn_readfirstlane(list[min(1, k - 1)]);
  __builtin_amdgcn_s_waitcnt(0);                 // Q fragments in (builtin, so the compiler knows)
  dma_tile(Kbh + (long long)j0 * K_TILE, k_lds, koff);
  wait_vm<0>();                                  // K(0)
  {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) sa[mt][nt][i] = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      bf16x8 a = k_frag(L, u);
      sa[u & 1][0] = mfma(a, qf[0][u >> 1], sa[u & 1][0]);
      sa[u & 1][1] = mfma(a, qf[1][u >> 1], sa[u & 1][1]);
    }
    wait_lds();
    if (k > 1) dma_tile(Kbh + (long long)j1 * K_TILE, k_lds, koff);
    dma_tile(Vbh + (long long)j0 * V_TILE, v_lds, voff);
    int nv0 = valid_slots(q, per_frame, j0);
    if (nv0 < BS) mask_pad_keys(sa, nv0, L.hh);
    float mx0 = max16(sa[1][0], max16(sa[0][0], -INFINITY));
    float mx1 = max16(sa[1][1], max16(sa[0][1], -INFINITY));
    st.mx[0] = fmaxf(mx0, __shfl_xor(mx0, 32));
    st.mx[1] = fmaxf(mx1, __shfl_xor(mx1, 32));
  }

  // ---- main loop, two tiles per trip so the two score buffers swap roles without copies
  int t = 0;
  int jn1 = j1;                                   // block of tile t+1
  for (; t + 2 < k; t += 2) {
    const int jn2 = __builtin_amdgcn_readfirstlane(list[t + 2]);
    const int jn3 = __builtin_amdgcn_readfirstlane(list[min(t + 3, k - 1)]);
    tile_step<true>(sa, sb, o, qf, st, L, Kbh + (long long)jn2 * K_TILE, true, Vbh + (long long)jn1 * V_TILE,
                    valid_slots(q, per_frame, jn1), k_lds, v_lds, koff, voff);
    tile_step<true>(sb, sa, o, qf, st, L, Kbh + (long long)jn3 * K_TILE, t + 3 < k, Vbh + (long long)jn2 * V_TILE,
                    valid_slots(q, per_frame, jn2), k_lds, v_lds, koff, voff);
    jn1 = jn3;
  }
  // here t is k-2 (two tiles left: t, t+1) or k-1 (one left); the scores of tile t are in sa
  if (t + 2 == k) {
    tile_step<true>(sa, sb, o, qf, st, L, Kbh, false, Vbh + (long long)jn1 * V_TILE, valid_slots(q, per_frame, jn1),
                    k_lds, v_lds, koff, voff);
    tile_step<false>(sb, sa, o, qf, st, L, Kbh, false, Vbh, BS, k_lds, v_lds, koff, voff);
  } else {
    tile_step<false>(sa, sb, o, qf, st, L, Kbh, false, Vbh, BS, k_lds, v_lds, koff, voff);
  }

  // ---- epilogue: normalise, convert, stage through LDS, write rows of 256 B
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float lt = st.l[nt] + __shfl_xor(st.l[nt], 32);
    const float inv = 1.0f / lt;
    if (lse && L.hh == 0) lse[qb * BS + 32 * nt + L.r] = st.m[nt] * kScale + __logf(lt);
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
        *(uint2*)(kl + (32 * nt + L.r) * O_STRIDE + (32 * dt + 8 * a + 4 * L.hh) * 2) = w;
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


// ==========================================================================================
// Shared-tile kernel: the four wavefronts of a workgroup own four query blocks at the same
// patch position in four consecutive frames.  Such blocks keep largely the same key blocks,
// so the workgroup walks the UNION of their four lists once, in ascending order, and every
// K/V tile of the union is brought into LDS once for all four (a ring of four 32 KB slots,
// filled three tiles ahead by direct-to-LDS loads that the four waves share out).  A wave
// computes on a tile only if its own list holds it.  One workgroup barrier per union tile
// keeps the ring consistent: it separates "everyone is done with tile u-1" from the refill of
// that slot, and "every share of tile u has landed" from its use.
//
// Inside a tile the 64 keys are taken as two online-softmax steps of 32 keys, so the vector
// ALU work of one half (max, exp, sum, pack) can run under the matrix-core work of the other:
//     S0 | S1 || softmax(S0) | PV0 || softmax(S1) | PV1
// ==========================================================================================
constexpr int RING = 4;
constexpr int SLOT = K_TILE + V_TILE;             // 32 KB
constexpr int RING_BYTES = RING * SLOT;           // 128 KB
constexpr int LDS_TOTAL = 160 * 1024;
constexpr int AUX_BYTES = LDS_TOTAL - RING_BYTES; // bitmaps + union list + counter

struct Soft2 {
  float m[2];     // reference max per query group (raw score units); -inf before the first tile
  float l[2];     // this lane's partial sum of probabilities
};

// Scheduling hints.  The matrix pipe and the vector ALU of a SIMD work at the same time only if
// the instruction stream of the (single) wave alternates between them, so the regions that
// hold two independent streams are closed with a pattern "1 matrix instruction, then V vector
// instructions", repeated; regions are fenced so that nothing drifts across.
__device__ __forceinline__ void region_fence() { __builtin_amdgcn_sched_barrier(0); }
template <int MFMAS, int VALU_PER>
__device__ __forceinline__ void interleave_pattern() {
#pragma unroll
  for (int i = 0; i < MFMAS; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // one MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);   // then VALU work
  }
}

// value of the other half-wave's lane (l ^ 32) combined by max: one v_permlane32_swap
__device__ __forceinline__ float max_across_halves(float x) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// row max of a 32-key half (two query groups) and the decision whether the reference max moves
__device__ __forceinline__ bool half_max(const f32x16& s0, const f32x16& s1, const Soft2& st, float& mx0, float& mx1) {
  mx0 = max_across_halves(max16(s0, -INFINITY));
  mx1 = max_across_halves(max16(s1, -INFINITY));
  // (mx - m) is NaN only when both are -inf (a half of pad keys before any real key): the
  // comparison is then false and nothing moves.
  return (mx0 - st.m[0]) * kC2 > kLazy || (mx1 - st.m[1]) * kC2 > kLazy;
}

// rare: move the reference max up and rescale what was accumulated against the old one
__device__ __forceinline__ void move_reference(f32x16 (&o)[4][2], Soft2& st, float mx0, float mx1, float& a0,
                                               float& a1) {
  const float n0 = fmaxf(st.m[0], mx0), n1 = fmaxf(st.m[1], mx1);
  a0 = st.m[0] == n0 ? 1.0f : __builtin_amdgcn_exp2f((st.m[0] - n0) * kC2);
  a1 = st.m[1] == n1 ? 1.0f : __builtin_amdgcn_exp2f((st.m[1] - n1) * kC2);
  st.m[0] = n0;
  st.m[1] = n1;
  st.l[0] *= a0;
  st.l[1] *= a1;
  acc_hazard_before();
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    scale_acc(o[dt][0], a0);
    scale_acc(o[dt][1], a1);
  }
  acc_hazard_after();
}

// probabilities already packed for the matrix cores, brought to a new reference (rare path)
__device__ __forceinline__ void scale_p(bf16x8& p, float a) {
#pragma unroll
  for (int i = 0; i < 8; i += 2) {
    f32x2 v = {(float)p[i] * a, (float)p[i + 1] * a};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    p[i] = b[0];
    p[i + 1] = b[1];
  }
}

// pad keys of one 32-key half: accumulator register i of half mt is key 32mt + 16(i>>3) + 8hh + (i&7)
__device__ __forceinline__ void mask_pad_half(f32x16& s0, f32x16& s1, int mt, int nv, int hh) {
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int key = 32 * mt + 16 * (i >> 3) + 8 * hh + (i & 7);
    if (key >= nv) {
      s0[i] = -INFINITY;
      s1[i] = -INFINITY;
    }
  }
}

// keep a score tile in ordinary vector registers (the softmax arithmetic reads it many times)
__device__ __forceinline__ void pin_vgpr(f32x16& x) { asm volatile("" : "+v"(x)); }

// One 64-key tile for one wave:  S0 | S1 || softmax(S0) | PV0 || softmax(S1) | PV1
// Operands are read from LDS one region ahead of the matrix instructions that use them (an LDS
// read takes on the order of a hundred cycles; requested just in time it would stall every
// matrix instruction).
struct TileOperands {
  bf16x8 k0[8], k1[8];   // K rows of keys 0..31 / 32..63, one per k-step over d
  bf16x8 va[8], vb[8];   // V^T rows: va = keys 0..31 (k-steps 0,1 x 4 channel groups), vb = keys 32..63
};

// All 32 operand reads of a tile are issued at once; the caller waits for them and can then
// hand the LDS slot back long before the arithmetic on the tile is finished.
__device__ __forceinline__ void fetch_tile_operands(TileOperands& x, const unsigned char* kread,
                                                    const unsigned char* vread, int ke, int ve) {
#pragma unroll
  for (int t = 0; t < 8; ++t) x.k0[t] = *(const bf16x8*)(kread + ((32 * t) ^ ke));
#pragma unroll
  for (int t = 0; t < 8; ++t) x.k1[t] = *(const bf16x8*)(kread + 32 * 256 + ((32 * t) ^ ke));
#pragma unroll
  for (int u = 0; u < 8; ++u) x.va[u] = *(const bf16x8*)(vread + (u & 3) * (32 * 128) + ((32 * (u >> 2)) ^ ve));
#pragma unroll
  for (int u = 0; u < 8; ++u) x.vb[u] = *(const bf16x8*)(vread + (u & 3) * (32 * 128) + ((32 * (2 + (u >> 2))) ^ ve));
}

template <typename Mid>
__device__ __forceinline__ void compute_shared_tile(const TileOperands& x, int hh, int nv, const bf16x8 (&qf)[2][8],
                                                    f32x16 (&o)[4][2], Soft2& st, Mid&& mid) {
  f32x16 s[2][2];
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 pf[2][4];
  const bf16x8 (&k0)[8] = x.k0;
  const bf16x8 (&k1)[8] = x.k1;
  const bf16x8 (&va)[8] = x.va;
  const bf16x8 (&vb)[8] = x.vb;
  float mx0, mx1;
  bool need;

  // ---- region 1: S0 = K[0..31] Q^T
  region_fence();
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    s[0][0] = mfma(k0[t], qf[0][t], t == 0 ? zero : s[0][0]);
    s[0][1] = mfma(k0[t], qf[1][t], t == 0 ? zero : s[0][1]);
  }
  pin_vgpr(s[0][0]);
  pin_vgpr(s[0][1]);
  region_fence();
  mid();           // a moment for ring housekeeping while the first scores drain from the matrix pipe
  if (nv < BS) mask_pad_half(s[0][0], s[0][1], 0, nv, hh);

  // ---- region 2: first quarter of S1 on the matrix cores, row max of S0 on the VALU
  region_fence();
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    s[1][0] = mfma(k1[t], qf[0][t], t == 0 ? zero : s[1][0]);
    s[1][1] = mfma(k1[t], qf[1][t], t == 0 ? zero : s[1][1]);
  }
  need = half_max(s[0][0], s[0][1], st, mx0, mx1);
  interleave_pattern<4, 6>();
  region_fence();
  if (__any(need)) {
    float a0, a1;
    move_reference(o, st, mx0, mx1, a0, a1);
  }

  // ---- region 3: rest of S1 on the matrix cores, exp / sum / pack of S0 on the VALU;
  //      the V operands of the first 32 keys are requested
  region_fence();
  {
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int t = 2; t < 8; ++t) {
      s[1][0] = mfma(k1[t], qf[0][t], s[1][0]);
      s[1][1] = mfma(k1[t], qf[1][t], s[1][1]);
    }
    exp_pack(s[0][0], st.m[0] * kC2, ls0, pf[0][0], pf[0][1]);
    exp_pack(s[0][1], st.m[1] * kC2, ls1, pf[1][0], pf[1][1]);
    st.l[0] += ls0;
    st.l[1] += ls1;
    interleave_pattern<12, 10>();
  }
  pin_vgpr(s[1][0]);
  pin_vgpr(s[1][1]);
  region_fence();
  if (nv < BS) mask_pad_half(s[1][0], s[1][1], 1, nv, hh);

  // ---- region 4: first quarter of PV0 on the matrix cores, row max of S1 on the VALU
  region_fence();
#pragma unroll
  for (int dt = 0; dt < 2; ++dt) {
    o[dt][0] = mfma(va[dt], pf[0][0], o[dt][0]);
    o[dt][1] = mfma(va[dt], pf[1][0], o[dt][1]);
  }
  need = half_max(s[1][0], s[1][1], st, mx0, mx1);
  interleave_pattern<4, 6>();
  region_fence();
  if (__any(need)) {
    // Everything accumulated so far, the four products above included, was formed against the
    // old reference and is rescaled; the probabilities of the first half still waiting in
    // registers for the rest of PV0 are brought to the new reference as well.
    float a0, a1;
    move_reference(o, st, mx0, mx1, a0, a1);
    scale_p(pf[0][0], a0);
    scale_p(pf[0][1], a0);
    scale_p(pf[1][0], a1);
    scale_p(pf[1][1], a1);
  }

  // ---- region 5: rest of PV0 on the matrix cores, exp / sum / pack of S1 on the VALU;
  //      the V operands of the last 32 keys are requested
  region_fence();
  {
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int dt = 2; dt < 4; ++dt) {
      o[dt][0] = mfma(va[dt], pf[0][0], o[dt][0]);
      o[dt][1] = mfma(va[dt], pf[1][0], o[dt][1]);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      o[dt][0] = mfma(va[4 + dt], pf[0][1], o[dt][0]);
      o[dt][1] = mfma(va[4 + dt], pf[1][1], o[dt][1]);
    }
    exp_pack(s[1][0], st.m[0] * kC2, ls0, pf[0][2], pf[0][3]);
    exp_pack(s[1][1], st.m[1] * kC2, ls1, pf[1][2], pf[1][3]);
    st.l[0] += ls0;
    st.l[1] += ls1;
    interleave_pattern<12, 10>();
  }
  region_fence();

  // ---- region 6: PV1
#pragma unroll
  for (int t = 2; t < 4; ++t)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      o[dt][0] = mfma(vb[4 * (t - 2) + dt], pf[0][t], o[dt][0]);
      o[dt][1] = mfma(vb[4 * (t - 2) + dt], pf[1][t], o[dt][1]);
    }
  region_fence();
  // every operand of this tile was in registers before region 6: the slot can be refilled
}

__global__ __launch_bounds__(256, 1) void attn_bf16_shared_kernel(Geo q, const unsigned char* __restrict__ Qp,
                                                                 const unsigned char* __restrict__ Kp,
                                                                 const unsigned char* __restrict__ Vt,
                                                                 const int32_t* __restrict__ idx,
                                                                 unsigned char* __restrict__ Op,
                                                                 float* __restrict__ lse, int dbg) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[LDS_TOTAL];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // Heads one after the other; inside a head a workgroup is one patch position and four
  // consecutive frames, and the frame groups of one position follow each other on one XCD
  // (workgroups are dealt round-robin to the 8 XCDs).
  const int per_frame = q.gh * q.gw;
  const int fgs = (q.T + 3) >> 2;
  const int pos_per_xcd = (per_frame + 7) >> 3;
  const int wg_per_head = 8 * pos_per_xcd * fgs;
  const long long bh = blockIdx.x / wg_per_head;
  const int n = blockIdx.x - (int)(bh * wg_per_head);
  const int xcd = n & 7, slot_id = n >> 3;
  const int pos = xcd + 8 * (slot_id / fgs);
  if (pos >= per_frame) return;                       // the whole workgroup leaves together
  const int f = 4 * (slot_id % fgs) + wave;
  const bool live = f < q.T;                          // a wave past the last frame only helps loading
  const long long qb = bh * q.g + (long long)min(f, q.T - 1) * per_frame + pos;
  const int k = q.k, g = q.g;

  unsigned* bitmap = (unsigned*)(smem + RING_BYTES);  // [4][bw]
  const int bw = (g + 31) >> 5;
  unsigned* ulist = bitmap + 4 * bw;                  // entries: key block | membership << 24
  unsigned* counter = (unsigned*)(smem + LDS_TOTAL - 16);
  int* ready = (int*)(smem + LDS_TOTAL - 64);         // [RING] union index whose tile the slot holds
  unsigned* passed = (unsigned*)(smem + LDS_TOTAL - 48);   // [RING] how many waves have left the slot, ever
  int* next_load = (int*)(smem + LDS_TOTAL - 32);     // next union entry nobody has requested yet
  int* freed = (int*)(smem + LDS_TOTAL - 28);         // union entries every wave has left (they leave in order)

  // ---- union of the four lists
  for (int i = threadIdx.x; i < 4 * bw; i += 256) bitmap[i] = 0u;
  if (threadIdx.x < RING) {
    ready[threadIdx.x] = -1;
    passed[threadIdx.x] = 0u;
  }
  if (threadIdx.x == 0) {
    *next_load = 0;
    *freed = 0;
  }
  __syncthreads();
  if (live) {
    const int32_t* list = idx + qb * k;
    for (int e = lane; e < k; e += 64) {
      int j = list[e];
      atomicOr(&bitmap[wave * bw + (j >> 5)], 1u << (j & 31));
    }
  }
  __syncthreads();
  if (wave == 0) {
    int cnt = 0;
    for (int base = 0; base < g; base += 64) {
      int j = base + lane;
      unsigned m4 = 0;
      if (j < g) {
#pragma unroll
        for (int w = 0; w < 4; ++w) m4 |= ((bitmap[w * bw + (j >> 5)] >> (j & 31)) & 1u) << w;
      }
      unsigned long long nz = __ballot(m4 != 0);
      int before = __builtin_amdgcn_mbcnt_hi((unsigned)(nz >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)nz, 0));
      if (m4) ulist[cnt + before] = (unsigned)j | (m4 << 24);
      cnt += __popcll(nz);
    }
    if (lane == 0) *counter = (unsigned)cnt;
  }
  __syncthreads();
  const int nU = __builtin_amdgcn_readfirstlane((int)*counter);

  // ---- per-lane constants
  const int r = lane & 31, hh = lane >> 5;
  const int krow = sigma(r);
  const int ke = (hh ^ (krow & 15)) << 4;
  const int ve = (hh ^ ((r >> 1) & 7)) << 4;
  const unsigned ring_lds = (unsigned)(uintptr_t)(lds_bytes)smem;
  unsigned koff[4], voff[4];
  tile_lane_offsets<256>(lane, koff);
  tile_lane_offsets<128>(lane, voff);
  const unsigned char* Kbh = Kp + bh * q.n_pad * (D * 2);
  const unsigned char* Vbh = Vt + bh * q.n_pad * (D * 2);
  // one wave brings a whole tile (K and V^T of union entry u) into ring slot u % RING
  auto issue_tile = [&](int u) {
    const unsigned e = ulist[u];
    const long long j = __builtin_amdgcn_readfirstlane((int)(e & 0xffffffu));
    const unsigned dst = ring_lds + (unsigned)(u & (RING - 1)) * SLOT;
    dma_tile(Kbh + j * K_TILE, dst, koff);
    dma_tile(Vbh + j * V_TILE, dst + K_TILE, voff);
  };
  // a tile this wave has requested becomes visible to the others once it has landed
  auto publish = [&](int& pending) {
    if (pending >= 0) {
      wait_vm<0>();
      if (lane == 0) __atomic_store_n(&ready[pending & (RING - 1)], pending, __ATOMIC_RELAXED);
      pending = -1;
    }
  };

  // Q fragments
  bf16x8 qf[2][8];
  {
    const unsigned char* qbase = Qp + (qb * BS) * (D * 2);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int t = 0; t < 8; ++t)
        qf[nt][t] = *(const bf16x8*)(qbase + (32 * nt + r) * (D * 2) + (16 * t + 8 * hh) * 2);
  }
  f32x16 o[4][2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][nt][i] = 0.f;
  Soft2 st;
  st.m[0] = st.m[1] = -INFINITY;
  st.l[0] = st.l[1] = 0.f;

  // Wait for the Q fragments with the builtin (not inline assembly) so that the compiler's own
  // counter bookkeeping knows they are in; otherwise it would wait for them again inside the
  // loop and drain the tile prefetch with them.  From here only tile loads are in flight.
  __builtin_amdgcn_s_waitcnt(0);
  // The ring is run without workgroup barriers.
  //   ready[s]   union entry whose tile slot s holds (set once the tile has landed)
  //   passed[s]  how many waves have ever left slot s; waves leave the entries in order, a wave
  //              leaves an entry as soon as its operand reads are done (or at once if its list
  //              does not hold the entry), and the wave that leaves last advances `freed`
  //   next_load  entries are requested strictly in order, entry L as soon as L < freed + RING;
  //              whichever wave notices first claims it with a compare-and-swap
  // A wave that is waiting for a tile is the natural one to request tiles: it has nothing else
  // to do, waits for the load to land and publishes it at once.  A busy wave only requests
  // when it passes by and nobody else has; it publishes after the tile it is about to compute.
  // Nobody can get more than RING entries ahead of the slowest wave, which keeps the counters
  // of successive uses of a slot apart.  Every wait is bounded: if a tile does not show up the
  // wave gives up (the output is then wrong, but the kernel always ends).
  int pending = -1;
  auto try_request = [&]() -> bool {
    const int L = __builtin_amdgcn_readfirstlane(__atomic_load_n(next_load, __ATOMIC_RELAXED));
    if (L >= nU) return false;
    const int fr = __builtin_amdgcn_readfirstlane(__atomic_load_n(freed, __ATOMIC_RELAXED));
    if (L >= fr + RING) return false;
    int got = L + 1;
    if (lane == 0) got = atomicCAS(next_load, L, L + 1);
    got = __builtin_amdgcn_readfirstlane(got);
    if (got != L) return false;
    publish(pending);                                 // at most one request of mine is in flight
    issue_tile(L);
    pending = L;
    return true;
  };
  const unsigned my_bit = live ? (1u << (24 + wave)) : 0u;
  bool gave_up = false;
  long long tc[6] = {0, 0, 0, 0, 0, 0};
  long long t_prev = (dbg & 4) ? __builtin_readcyclecounter() : 0;
#define TICK(c) if (dbg & 4) { long long t_now = __builtin_readcyclecounter(); tc[c] += t_now - t_prev; t_prev = t_now; }
  for (int u = 0; u < nU && !gave_up; ++u) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      pin_acc(o[dt][0]);
      pin_acc(o[dt][1]);
    }
    const int slot_i = u & (RING - 1);
    if (!(dbg & 2)) {
      try_request();
      int spins = 0;
      while (__builtin_amdgcn_readfirstlane(__atomic_load_n(&ready[slot_i], __ATOMIC_RELAXED)) != u) {
        if (pending >= 0) {
          long long t_a = (dbg & 4) ? __builtin_readcyclecounter() : 0;
          publish(pending);                           // idle: wait for my own request and hand it over
          if (dbg & 4) { tc[4] += __builtin_readcyclecounter() - t_a; tc[5] += 1; }
        } else if (!try_request()) {
          __builtin_amdgcn_s_sleep(2);
          if (++spins > (1 << 20)) {
            gave_up = true;
            break;
          }
        }
      }
      if (gave_up) break;
    }
    TICK(0)
    const unsigned e = __builtin_amdgcn_readfirstlane(ulist[u]);
    const bool mine = (e & my_bit) && !(dbg & 1);
    TileOperands x;
    if (mine) {
      const unsigned char* slot = smem + slot_i * SLOT;
      fetch_tile_operands(x, slot + krow * 256, slot + K_TILE + r * 128, ke, ve);
    }
    if (!(dbg & 2)) {
      wait_lds();                                    // my reads of the slot are complete: hand it back
      unsigned old = 0;
      if (lane == 0) {
        old = atomicAdd(&passed[slot_i], 1u);
        if (old + 1 == 4u * (unsigned)((u >> 2) + 1)) __atomic_store_n(freed, u + 1, __ATOMIC_RELAXED);
      }
    }
    TICK(1)
    if (mine) {
      const int j = (int)(e & 0xffffffu);
      const int nv = valid_slots(q, per_frame, j);
      compute_shared_tile(x, hh, nv, qf, o, st, [&]() {
        if (!(dbg & 2)) publish(pending);             // my request from the top of this trip has had time to land
      });
      TICK(2)
    }
  }
  publish(pending);
  if ((dbg & 4) && lse && lane == 0) {
    long long wid = (long long)blockIdx.x * 4 + wave;
    for (int c = 0; c < 6; ++c) lse[wid * 6 + c] = (float)tc[c];
  }
  __syncthreads();                                    // everyone is done with the ring: reuse it to stage the output
  if (!live) return;

  unsigned char* stage = smem + wave * SLOT;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float lt = st.l[nt] + __shfl_xor(st.l[nt], 32);
    const float inv = 1.0f / lt;
    if (lse && hh == 0 && !(dbg & 4)) lse[qb * BS + 32 * nt + r] = st.m[nt] * kScale + __logf(lt);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        f32x2 v0 = {o[dt][nt][4 * a] * inv, o[dt][nt][4 * a + 1] * inv};
        f32x2 v1 = {o[dt][nt][4 * a + 2] * inv, o[dt][nt][4 * a + 3] * inv};
        bf16x2 b0 = __builtin_convertvector(v0, bf16x2);
        bf16x2 b1 = __builtin_convertvector(v1, bf16x2);
        uint2 w2 = make_uint2(*(unsigned*)&b0, *(unsigned*)&b1);
        *(uint2*)(stage + (32 * nt + r) * O_STRIDE + (32 * dt + 8 * a + 4 * hh) * 2) = w2;
      }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  unsigned char* obase = Op + (qb * BS) * (D * 2);
#pragma unroll
  for (int it = 0; it < 16; ++it) {
    int row = it * 4 + (lane >> 4), ch = lane & 15;
    *(uint4*)(obase + row * (D * 2) + ch * 16) = *(const uint4*)(stage + row * O_STRIDE + ch * 16);
  }
}

hipError_t launch_attn_bf16(const Geo& q, const void* Qp, const void* Kp, const void* Vt, const int32_t* idx, void* Op,
                            float* lse, hipStream_t s) {
  const int per_frame = q.gh * q.gw;
  // DA_ATTN_KERNEL=private selects the kernel in which every wave streams its own tiles (the
  // fallback when the union bookkeeping of the shared-tile kernel does not fit in LDS).
  const char* env = getenv("DA_ATTN_KERNEL");
  bool want_private = env && strcmp(env, "private") == 0;
  long long union_max = (long long)q.g < 4LL * q.k ? q.g : 4LL * q.k;
  long long aux = 4LL * 4 * ((q.g + 31) / 32) + 4 * union_max + 64;
  if (!want_private && aux <= AUX_BYTES && q.g < (1 << 24)) {
    unsigned grid = (unsigned)((long long)q.B * q.H * 8 * ((per_frame + 7) / 8) * ((q.T + 3) / 4));
    hipLaunchKernelGGL(attn_bf16_shared_kernel, dim3(grid), dim3(256), 0, s, q, (const unsigned char*)Qp,
                       (const unsigned char*)Kp, (const unsigned char*)Vt, idx, (unsigned char*)Op, lse,
                       getenv("DA_ATTN_DBG") ? atoi(getenv("DA_ATTN_DBG")) : 0);
    return hipGetLastError();
  }
  long long total_qb = (long long)q.B * q.H * q.g;
  long long wgs = (total_qb + 3) / 4;
  int wg_per_xcd = (int)((wgs + 7) / 8);
  unsigned grid = (unsigned)((long long)q.B * q.H * 8 * ((per_frame + 7) / 8) * ((q.T + 3) / 4));
  hipLaunchKernelGGL(attn_bf16_kernel, dim3(grid), dim3(256), 0, s, q, (const unsigned char*)Qp,
                     (const unsigned char*)Kp, (const unsigned char*)Vt, idx, (unsigned char*)Op, lse, wg_per_xcd,
                     total_qb, 1);
  return hipGetLastError();
}

}  // namespace da
