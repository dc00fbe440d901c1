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
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[dt][nt][i] *= alpha;
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
  dma_tile(Kbh + (long long)j0 * K_TILE, k_lds, koff);
  wait_vm<0>();                                  // Q fragments and K(0)
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

hipError_t launch_attn_bf16(const Geo& q, const void* Qp, const void* Kp, const void* Vt, const int32_t* idx, void* Op,
                            float* lse, hipStream_t s) {
  long long total_qb = (long long)q.B * q.H * q.g;
  long long wgs = (total_qb + 3) / 4;
  int wg_per_xcd = (int)((wgs + 7) / 8);
  unsigned grid = (unsigned)(wg_per_xcd * 8);
  const char* env = getenv("DA_ATTN_MAP");
  int map_mode = env ? atoi(env) : 1;
  if (map_mode != 0) {
    int per_frame = q.gh * q.gw;
    grid = (unsigned)((long long)q.B * q.H * 8 * ((per_frame + 7) / 8) * ((q.T + 3) / 4));
  }
  hipLaunchKernelGGL(attn_bf16_kernel, dim3(grid), dim3(256), 0, s, q, (const unsigned char*)Qp,
                     (const unsigned char*)Kp, (const unsigned char*)Vt, idx, (unsigned char*)Op, lse, wg_per_xcd,
                     total_qb, map_mode);
  return hipGetLastError();
}

}  // namespace da
