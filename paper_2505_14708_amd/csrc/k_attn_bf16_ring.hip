// SparseAttn for bf16 storage, d = 128, blocks of 64 or 128 tokens, on the CDNA4 matrix cores
// (v_mfma_f32_32x32x16_bf16, float32 accumulation): the shared-ring kernel.  (Described for
// 64-token blocks; what changes for 128 is said at the kernel.)
//
// Why tiles are shared.  With 64 queries against a 64-key tile the arithmetic intensity is
// 64 flop per byte of K/V, far below the machine balance, and a kernel in which every query
// block streams its own tiles is bound by the memory fabric.  Query blocks at the same patch
// position in consecutive frames keep largely the same key blocks, so a workgroup takes four
// such blocks and walks the UNION of their lists once: every K tile of the union is brought
// into LDS once for all four, and the V tiles they fetch meet in L2.
//
// Workgroup = 8 wavefronts, two per SIMD.  A wavefront owns 32 queries (half a block): with
// half the accumulators a wave fits in 256 registers, two waves share a SIMD, and while one is
// in its softmax (vector ALU) the other keeps the matrix pipe busy; the same pairing hides LDS
// latency and the waits of the ring protocol.  The two waves of a SIMD belong to different
// query blocks so that they are rarely in the same phase.
//
// Per key tile a wave computes
//     S^T = K Q^T      (64 keys x 32 queries: 2 MFMA tiles of 32x32, 8 k-steps over d)
//     online softmax over the 64 keys
//     O^T += V^T P^T   (128 channels x 32 queries: 4 MFMA tiles, 4 k-steps over the keys)
// The transposed forms put the query on the lane axis (lane l holds query l%32), so row max and
// row sum run down a lane's own registers plus one exchange between lanes l and l^32.  Lane l
// feeds K row sigma(l%32) (sigma swaps bits 2 and 3): then the scores a lane holds in
// accumulator registers 8t..8t+7 belong to keys 16t + 8*(l/32) + 0..7, exactly the eight
// contraction elements the P^T operand of the second product needs, so P goes from accumulator
// to operand without leaving the lane.  V arrives from the reorder step transposed and cut into
// these operands (one product step's 64 operands are one contiguous KB), so K rows are read from
// LDS, and V^T operands from global memory, as plain 16-byte pieces.
//
// The ring.  Eight 16 KB slots, each one K tile.  Tiles travel HBM/L2 -> LDS by 16-byte
// direct-to-LDS loads; the lane that writes LDS position p of row r fetches global chunk
// p ^ swizzle(r), which makes the operand reads conflict-free.  There are no workgroup barriers
// in the tile loop:
//   ready[s]   union entry whose K tile slot s holds (set once the tile has landed)
//   left[s]    how many waves have yet to read the tile in slot s (set when the tile is asked for: the
//              live waves of the query blocks that hold the entry; every reader takes one off when it
//              is through): at zero the slot may be overwritten
//   next_load  entries are requested strictly in order, entry L once its slot L % 8 is free, by the waves
//              that are waiting for a tile: the one that notices first claims it with a compare-and-
//              swap, waits for the load (it is idle anyway, or at the top of its next trip) and
//              publishes it.  Waves that have a tile to work on do not look for room.
// A wave reads all of this with one LDS access per poll.  Every wait is bounded: if a tile does
// not show up the wave gives up (its output rows are then NaN, but the kernel always ends).
//
// V does not go through LDS.  After S = QK^T of a tile a wave knows the largest score of each of
// its queries; when every score of the tile is so far below the best the query has seen that
// all such keys of a row together weigh less than 2^-14 of its largest term, the tile cannot
// change the result at the precision of the output and its exponentials and second product are
// skipped.  With peaked attention that is the common case, so V^T operands are fetched from
// global memory (L2) straight into registers, only by the waves that need them, while the
// exponentials are being computed.
//
// The normaliser of a row is the sum of its probabilities as the second product sees them, i.e. after their
// rounding to bf16 (v_dot2c_f32_bf16 with a pair of ones: one instruction per two probabilities): numerator and
// denominator then carry the same rounding, and a row dominated by one key returns that key's V row exactly.
//
// The running max only moves (and O is rescaled) when a row max exceeds it by more than 2^8 in
// the exponent's units; until then probabilities are formed against the stale max, which is
// exact after the final division because numerator and denominator share it.
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include "da_internal.h"

namespace da {
namespace ring {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) unsigned char* lds_bytes;

constexpr int D = 128;
constexpr int BS = 64;
constexpr int K_TILE = BS * D * 2;   // 16 KB, rows of 256 B
constexpr int V_TILE = D * BS * 2;   // 16 KB, rows of 128 B
constexpr int RING = 8;
constexpr int SLOT = K_TILE;
constexpr int RING_BYTES = RING * SLOT;           // 128 KB
constexpr int LDS_TOTAL = 160 * 1024;
constexpr int AUX_BYTES = LDS_TOTAL - RING_BYTES; // bitmaps + union list + ring state
constexpr int WAVES = 8;
constexpr int O_STRIDE = D * 2 + 16;              // padded row stride of the output staging area
constexpr float kScale = 0.08838834764831845f;                      // 1/sqrt(128)
constexpr float kC2 = 0.08838834764831845f * 1.4426950408889634f;   // log2(e)/sqrt(128)
constexpr float kLazy = 8.0f;                     // move the running max only past this many powers of two
constexpr float kDropLog2 = 14.0f;                // all keys dropped from a row together weigh less than 2^-14 of its largest term
constexpr int kSpinLimit = 1 << 20;

// Waves whose bounded wait for a tile ran out since the library was loaded (their rows were written as NaN).
// No valid input makes that happen; the host can ask (da_wait_failures).
__device__ unsigned long long g_wait_failures = 0ull;

// ---------------------------------------------------------------------------------- tile movement
// 16 KB tile, rows of ROWB bytes, moved 1 KB (64 lanes x 16 B) per step; step `it` covers rows
// it*RPS .. it*RPS+RPS-1 (RPS*ROWB = 1024), so global and LDS offsets are both it*1024 plus a
// per-lane part that only depends on it & 3.
template <int ROWB>
__device__ inline void tile_lane_offsets(int lane, unsigned loff[4]) {
  constexpr int CPR = ROWB / 16;
  constexpr int RPS = 64 / CPR;
  const int r_in = lane / CPR, p = lane % CPR;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    int row = a * RPS + r_in;
    int sw = ROWB == 256 ? (row & 15) : ((row >> 1) & 7);
    loff[a] = r_in * ROWB + ((p ^ sw) << 4);
  }
}

// Direct-to-LDS load of 16 bytes per lane: lane i's data lands at m0 + 16*i.  m0 is put back afterwards (the
// load has read it by then), so whatever the compiler keeps in it across this statement survives.
__device__ __forceinline__ void dma16(const unsigned char* g, unsigned lds_addr) {
  unsigned keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
      : "=&s"(keep)
      : "v"(g), "s"(lds_addr)
      : "memory");
}
__device__ __forceinline__ void dma_tile(const unsigned char* src, unsigned lds_addr, const unsigned (&loff)[4]) {
#pragma unroll
  for (int it = 0; it < 16; ++it) dma16(src + it * 1024 + loff[it & 3], lds_addr + it * 1024);
}
__device__ __forceinline__ void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ inline int sigma(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------- softmax pieces
__device__ __forceinline__ float max16(const f32x16& a, float m) {
#pragma unroll
  for (int i = 0; i < 16; i += 2) m = fmaxf(fmaxf(a[i], a[i + 1]), m);   // v_max3_f32
  return m;
}

// max with the other half-wave's lane (l ^ 32): one v_permlane32_swap
__device__ __forceinline__ float max_across_halves(float x) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// exp / sum / pack of 16 scores (one accumulator tile) into two P operands
__device__ __forceinline__ void exp_pack(const f32x16& s, float mc, float& lsum, bf16x8& p_lo, bf16x8& p_hi) {
  const bf16x2 kOnes = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], kC2, -mc));
    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 1], kC2, -mc));
    f32x2 pp = {p0, p1};
    bf16x2 pb = __builtin_convertvector(pp, bf16x2);
    lsum = __builtin_amdgcn_fdot2_f32_bf16(pb, kOnes, lsum, false);   // the sum of what the second product sees
    if (i < 8) {
      p_lo[i] = pb[0];
      p_lo[i + 1] = pb[1];
    } else {
      p_hi[i - 8] = pb[0];
      p_hi[i - 7] = pb[1];
    }
  }
}

// pad keys out of the softmax: accumulator register i of half mt is key 32mt + 16(i>>3) + 8hh + (i&7)
__device__ __forceinline__ void mask_pad_half(f32x16& s, int mt, int nv, int hh) {
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int key = 32 * mt + 16 * (i >> 3) + 8 * hh + (i & 7);
    if (key >= nv) s[i] = -INFINITY;
  }
}

// n / d for 0 <= n < 2^24, d >= 1, by way of the float reciprocal (exact: the estimate is off by one at most)
__device__ __forceinline__ int small_div(int n, int d) {
  int qt = (int)((float)n * __frcp_rn((float)d));
  const int rem = n - qt * d;
  qt += rem >= d ? 1 : 0;
  qt -= rem < 0 ? 1 : 0;
  return qt;
}

// valid slots of block j (blocks are numbered below 2^22)
__device__ __forceinline__ int valid_slots(const Geo& q, int per_frame, int j) {
  const int rr = j - small_div(j, per_frame) * per_frame;
  const int bi = small_div(rr, q.gw), bj = rr - bi * q.gw;
  return min(q.ph, q.fh - bi * q.ph) * min(q.pw, q.fw - bj * q.pw);
}

struct Soft {
  float m;     // reference max (raw score units); -inf before the first tile
  float top;   // largest score seen so far (the reference trails it by at most kLazy powers of two)
  float l;     // this lane's partial sum of probabilities
};

// One 64-key tile for one wave (32 queries).  kaddr[t] is this lane's LDS address of the K
// operand of k-step t (swizzle already applied; the second 32 keys sit 8 KB further).  vt is
// this lane's 16 bytes of the first operand group of the tile's V^T in global memory (operand
// order: the 64 lanes' operands of (k-step t, channel group dt) are the contiguous KB number
// 4t + dt of the tile, so every load of a wave is one contiguous KB).
__device__ __forceinline__ bool compute_tile(const unsigned char* const (&kaddr)[8], const unsigned char* vt, int hh,
                                             int nv, bool pad_query, float skip, const bf16x8 (&qf)[8],
                                             f32x16 (&o)[4], Soft& st) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 s0, s1;
  bf16x8 va[4][4];
  {
    // S^T = K Q^T; all sixteen K operands are asked for before the first product, so the LDS
    // latency is paid once per tile
    bf16x8 ka[8], kb[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      ka[t] = *(const bf16x8*)(kaddr[t]);
      kb[t] = *(const bf16x8*)(kaddr[t] + 32 * 256);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      s0 = mfma(ka[t], qf[t], t == 0 ? zero : s0);
      s1 = mfma(kb[t], qf[t], t == 0 ? zero : s1);
    }
  }
  if (nv < BS) {
    mask_pad_half(s0, 0, nv, hh);
    mask_pad_half(s1, 1, nv, hh);
  }
  // online softmax over the 64 keys
  const float mx = max_across_halves(max16(s1, max16(s0, -INFINITY)));   // finite: slot 0 of a block is valid
  // A key whose score is more than `skip` powers of two below the query's best score so far
  // weighs less than 2^-skip of that query's largest term, in the normaliser and in the output.
  // skip = log2(keys in the row) + kDropLog2, so whatever is dropped from a row adds up to less
  // than 2^-kDropLog2 of that term: below the resolution of a bf16 result at any sequence length.
  // When every key of the tile is that small for all 32 queries, the exponentials and the second
  // product are skipped.  (Never the first time: top is -inf.)  Pad query slots have no say: their
  // rows are zero, every score is 0, and nobody reads their output.
  if (__all(pad_query || (mx - st.top) * kC2 < -skip)) return false;
  // V^T operands: on their way while the exponentials are computed.  (Asking for them before the first product
  // where tiles keep mattering was tried: a tile dropped after all then leaves loads in flight, the compiler has
  // to wait for everything outstanding at the top of every tile, the ring's transfers included, and the common
  // case lost more than the other gained.)
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) va[t][dt] = *(const bf16x8*)(vt + (t * 4 + dt) * 1024);
  st.top = fmaxf(st.top, mx);
  if (__any((mx - st.m) * kC2 > kLazy)) {
    const float m_new = fmaxf(st.m, mx);
    const float alpha = st.m == m_new ? 1.0f : __builtin_amdgcn_exp2f((st.m - m_new) * kC2);   // 0 the first time
    st.m = m_new;
    st.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
  }
  bf16x8 pf[4];
  float ls = 0.f;
  const float mc = st.m * kC2;
  exp_pack(s0, mc, ls, pf[0], pf[1]);
  exp_pack(s1, mc, ls, pf[2], pf[3]);
  st.l += ls;
  // O^T += V^T P^T
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = mfma(va[t][dt], pf[t], o[dt]);
  return true;
}

// How the frames that do not fill a group of `fg` are spread over workgroups.
struct TailPlan {
  int full_groups;   // groups of fg frames
  int rem;           // frames left over (0: no tail workgroups)
  int per_wg;        // positions per tail workgroup
  int tail_wgs;      // tail workgroups per head
};
__host__ __device__ inline TailPlan tail_plan(const Geo& q, int fg) {
  TailPlan p;
  p.full_groups = q.T / fg;
  p.rem = q.T - p.full_groups * fg;
  p.per_wg = p.rem ? fg / p.rem : 1;
  const int per_frame = q.gh * q.gw;
  p.tail_wgs = p.rem ? (per_frame + p.per_wg - 1) / p.per_wg : 0;
  return p;
}

// SUB = 64-token sub-blocks per block (1: 8x8 patches, 2: 128-token blocks such as 8x16 patches).  A block of
// 128 is two K tiles and two V tiles in a row, and its queries are four waves' worth: the workgroup then takes two
// query blocks (two consecutive frames) instead of four, and a key block enters the union walk as two entries.
// LISTS: the kept blocks come as lists of any length (row_ptr) instead of k per row.
template <int SUB, bool LISTS>
__global__ __launch_bounds__(512, 2) void attn_bf16_ring_kernel(Geo q, const unsigned char* __restrict__ Qp,
                                                               const unsigned char* __restrict__ Kp,
                                                               const unsigned char* __restrict__ Vt,
                                                               const int32_t* __restrict__ idx,
                                                               const int32_t* __restrict__ row_ptr, long long cap,
                                                               unsigned char* __restrict__ Op, float* __restrict__ lse,
                                                               int balance, float skip, int direct,
                                                               unsigned long long* __restrict__ tile_counts) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[LDS_TOTAL];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // Heads one after the other (the K/V of the heads in flight then fit the last-level cache);
  // inside a head a workgroup is one patch position and FG consecutive frames, and the frame
  // groups of one position follow each other on one XCD (workgroups are dealt round-robin to the
  // 8 XCDs).
  constexpr int FG = 4 / SUB;                         // query blocks (frames) per workgroup
  constexpr int BLOCK = BS * SUB;                     // slots per block
  // The frames that do not fill a group (T mod FG of them) are taken position by position into
  // workgroups of their own, FG / (T mod FG) positions each: their lists have little in common, but
  // a workgroup with one live query block out of four would cost as much as a full one.
  const int per_frame = q.gh * q.gw;
  const TailPlan plan = tail_plan(q, FG);
  const int fgs = plan.full_groups;
  const int pos_per_xcd = (per_frame + 7) >> 3;
  const int regular = 8 * pos_per_xcd * fgs;
  const int wg_per_head = regular + plan.tail_wgs;
  const long long bh = blockIdx.x / wg_per_head;
  // the tail workgroups (longer walks) come first within a head, the regular ones after them
  const int n = blockIdx.x - (int)(bh * wg_per_head) - plan.tail_wgs;   // < 0: tail workgroup n + tail_wgs
  // waves w and w+4 share a SIMD: give them different query blocks.  part = which 32 queries of the block.
  const int half = wave >> 2;
  const int qblk = SUB == 1 ? (wave + 2 * half) & 3 : half;
  const int part = SUB == 1 ? half : wave & 3;
  // query block w of this workgroup: (position, frame), or none
  // (divisions of small non-negative numbers: by way of the float reciprocal)
  const int n_over_fgs = n >= 0 ? small_div(n >> 3, max(fgs, 1)) : 0;
  auto slot_pos = [&](int w) -> int {
    if (n >= 0) return (n & 7) + 8 * n_over_fgs;
    return w < plan.per_wg * plan.rem ? (n + plan.tail_wgs) * plan.per_wg + small_div(w, plan.rem) : per_frame;
  };
  auto slot_frame = [&](int w) -> int {
    if (n >= 0) return FG * ((n >> 3) - n_over_fgs * fgs) + w;
    return fgs * FG + (w - small_div(w, plan.rem) * plan.rem);
  };
  // block number of query block w, -1 if the slot is empty
  auto slot_block = [&](int w) -> int {
    const int p = slot_pos(w), fr = slot_frame(w);
    return p < per_frame && fr < q.T ? fr * per_frame + p : -1;
  };
  if (n >= 0 && slot_pos(0) >= per_frame) return;     // a regular workgroup past the last position: all of it leaves
  const int my_block = slot_block(qblk);
  const bool has_block = my_block >= 0;
  // a wave without a query block, or whose 32 slots of it are all pad slots, only helps with the ring
  const bool live = has_block && 32 * part < block_valid(q, has_block ? my_block : 0);
  const int pos = has_block ? slot_pos(qblk) : 0;
  const long long qb = bh * q.g + (has_block ? my_block : 0);
  const int g = q.g;
  // The list of my query block: k columns at idx + (row) * k, or, with row_ptr (lists of any length, one head's
  // after the other in a stretch of `cap` entries), the columns between two offsets.
  int k = q.k;
  const int32_t* list = idx + qb * k;
  if (LISTS) {
    const int32_t* rp = row_ptr + bh * (g + 1) + (has_block ? my_block : 0);
    // (offsets that are not what the interface asks for are brought into the head's stretch: such lists give
    // unspecified results, but nothing outside the arrays is read)
    const int begin = min(max(rp[0], 0), (int)cap);
    list = idx + bh * cap + begin;
    k = min(max(rp[1] - begin, 0), (int)cap - begin);
    // the cut of the drop rule goes by the number of keys in this row
    skip = log2f((float)max(k, 1) * (float)BLOCK) + kDropLog2;
  }

  // Q fragments (B operand): lane (query r, half-wave hh) holds d = 16t + 8hh .. +7.  Asked for
  // first, so that they arrive while the lists are being merged.
  // With `direct`, Qp and Op are the caller's Q and O (q.in, q.out: in the original token order as a rule): the
  // reordering of Q and the restoring of O (Algorithms 1 and 2) are then this kernel's addressing, slot -> row.
  const BlockPos qpos = block_pos(q, has_block ? my_block : 0);
  const long long q_first = block_first_row(q, has_block ? my_block : 0, qpos);
  const int q_pitch = block_row_pitch(q, qpos);
  // byte offset of the row of slot s of my query block in Qp / Op, or -1 (a pad slot has no row of its own there)
  auto row_bytes = [&](int s, const Rows& where) -> long long {
    if (!direct) return (qb * BLOCK + s) * (long long)(D * 2);
    if (s >= qpos.vh * qpos.vw) return -1;
    const int u = s / qpos.vw, v = s - u * qpos.vw;
    return row_offset(where, q.H, bh, q_first + (long long)u * q_pitch + v) * 2;
  };
  bf16x8 qf[8];
  {
    const int r = lane & 31, hh = lane >> 5;
    const long long row = row_bytes(32 * part + r, q.in);
    const unsigned char* qrow = Qp + max(row, 0LL);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      qf[t] = *(const bf16x8*)(qrow + (16 * t + 8 * hh) * 2);
      if (row < 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) qf[t][i] = (__bf16)0.f;
      }
    }
  }

  unsigned* bitmap = (unsigned*)(smem + RING_BYTES);  // [FG][bw] one bitmap of kept key blocks per query block
  const int bw = (g + 31) >> 5;
  unsigned* ulist = bitmap + 4 * bw;                  // union entries: key sub-block | (valid slots - 1) << 22 | membership << 28
  const int union_max = SUB * (LISTS ? g : min(g, FG * q.k));
  int* ctrl = (int*)(smem + LDS_TOTAL - 128);         // [32]: ready[8], left[8], next_load, count, n_own, ..., live waves
  int* ready = ctrl;                                  // [RING]
  int* left = ctrl + 8;                               // [RING]
  int* next_load = ctrl + 16;
  int* count = ctrl + 17;                             // [2]

  // ---- union of the workgroup's lists (the first 256 entries of a list are asked for before the
  // bitmaps are cleared, so that the two latencies overlap)
  const bool lister = live && part == 0;              // the wave that brings in the list of its query block
  int pre[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) pre[i] = lister && lane + 64 * i < k ? list[lane + 64 * i] : -1;
  for (int i = threadIdx.x; i < 4 * bw; i += 512) bitmap[i] = 0u;
  if (threadIdx.x < 32) ctrl[threadIdx.x] = threadIdx.x < RING ? -1 : 0;
  __syncthreads();
  if (live && lane == 0) atomicOr(&ctrl[28], 1 << wave);   // which waves take tiles at all
  if (lister) {
    // (an entry that is no block number is left out: it must not reach the bitmap, let alone an address)
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if ((unsigned)pre[i] < (unsigned)g) atomicOr(&bitmap[qblk * bw + (pre[i] >> 5)], 1u << (pre[i] & 31));
    for (int e = lane + 256; e < k; e += 64) {
      int j = list[e];
      if ((unsigned)j < (unsigned)g) atomicOr(&bitmap[qblk * bw + (j >> 5)], 1u << (j & 31));
    }
  }
  __syncthreads();
  // The workgroup's own blocks go first (when kept): a query's best scores tend to be
  // there, and the sooner the running maximum is near its final value, the more of the other
  // tiles turn out negligible.
  int own_j[FG];                                      // the workgroup's own blocks (-1: empty slot)
#pragma unroll
  for (int w = 0; w < FG; ++w) own_j[w] = slot_block(w);
  // membership of key block j in the workgroup's lists (0 for the own blocks unless asked for)
  auto membership = [&](int j, bool want_own) -> unsigned {
    bool own = false;
#pragma unroll
    for (int w = 0; w < FG; ++w) own = own || j == own_j[w];
    unsigned m4 = 0;
    if (j < g && own == want_own) {
#pragma unroll
      for (int w = 0; w < FG; ++w) m4 |= ((bitmap[w * bw + (j >> 5)] >> (j & 31)) & 1u) << w;
    }
    return m4;
  };
  // a key block becomes one entry per 64-slot sub-block that holds a valid slot (in a row)
  auto second = [&](int j) -> bool { return SUB == 2 && j < g && valid_slots(q, per_frame, j) > BS; };
  auto put_entries = [&](int at, int j, unsigned m4, bool two) {
    const int nvb = valid_slots(q, per_frame, j);
    ulist[at] = (unsigned)(j * SUB) | ((unsigned)(min(nvb, BS) - 1) << 22) | (m4 << 28);
    if (two) ulist[at + 1] = (unsigned)(j * SUB + 1) | ((unsigned)(nvb - BS - 1) << 22) | (m4 << 28);
  };
  auto lanes_before = [&](unsigned long long m) -> int {
    return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0));
  };
  // every wave takes a contiguous eighth of the key blocks, 64 at a time: count, then place
  int* wcount = ctrl + 20;                            // [WAVES]
  const int chunks = (g + 63) >> 6, cpw = (chunks + WAVES - 1) / WAVES;
  const int c_lo = wave * cpw, c_hi = min(chunks, c_lo + cpw);
  {
    int cnt = 0;
    if (SUB == 1) {
      // one entry per key block in any list: count the bits of the OR of the bitmaps, word by word
      // (lane l takes word l of the wave's range), minus the own blocks among them
      const int w_lo = 2 * c_lo, w_hi = min(2 * c_hi, bw);
      for (int base = w_lo; base < w_hi; base += 64) {
        const int word = base + lane;
        unsigned v = 0u;
        if (word < w_hi) {
#pragma unroll
          for (int w = 0; w < FG; ++w) v |= bitmap[w * bw + word];
#pragma unroll
          for (int w = 0; w < FG; ++w)
            if (own_j[w] >= 0 && (own_j[w] >> 5) == word) v &= ~(1u << (own_j[w] & 31));
        }
        int pop = __popc(v);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) pop += __shfl_xor(pop, o);
        cnt += pop;
      }
    } else {
      for (int c = c_lo; c < c_hi; ++c) {
        const int j = c * 64 + lane;
        const bool in = membership(j, false) != 0u;
        cnt += __popcll(__ballot(in)) + __popcll(__ballot(in && second(j)));
      }
    }
    if (lane == 0) wcount[wave] = cnt;
    if (wave == 0) {
      int j = -1;
#pragma unroll
      for (int w = 0; w < FG; ++w) j = lane == w ? own_j[w] : j;
      const unsigned m4 = j >= 0 ? membership(j, true) : 0u;
      const bool two = m4 != 0u && second(j);
      const unsigned long long nz = __ballot(m4 != 0u), n2 = __ballot(two);
      if (m4) put_entries(lanes_before(nz) + lanes_before(n2), j, m4, two);
      if (lane == 0) count[1] = __popcll(nz) + __popcll(n2);
    }
  }
  __syncthreads();
  {
    int at = count[1];
    for (int w = 0; w < wave; ++w) at += wcount[w];
    for (int c = c_lo; c < c_hi; ++c) {
      const int j = c * 64 + lane;
      const unsigned m4 = membership(j, false);
      const bool two = m4 != 0u && second(j);
      const unsigned long long nz = __ballot(m4 != 0u), n2 = __ballot(two);
      if (m4) put_entries(at + lanes_before(nz) + lanes_before(n2), j, m4, two);
      at += __popcll(nz) + __popcll(n2);
    }
    if (wave == WAVES - 1 && lane == 0) count[0] = at;
  }
  __syncthreads();
  const int nU = __builtin_amdgcn_readfirstlane(count[0]);
  const int n_own = __builtin_amdgcn_readfirstlane(count[1]);

  // ---- order of the walk.  In ascending order the four blocks' shares of the work come in
  // runs (the earliest frames of the union only matter to the first block, the latest only to
  // the last), and since nobody can run more than RING entries ahead, waves would take turns
  // waiting.  Entries with the same membership form a class (15 classes); each class is spread
  // evenly over the walk: the p-th of c entries of a class gets the key (2p+1)/(2c), and the
  // walk goes by ascending key.  Every stretch of the walk then holds every block's fair share.
  // The softmax does not care about the order of the keys.  (Skipped when the two extra
  // arrays it needs do not fit in LDS; the walk is then in ascending order.)
  if (balance) {
    unsigned* rest = ulist + n_own;                   // the own blocks keep their place in front
    const int nR = nU - n_own;
    unsigned* upos = ulist + union_max;               // position of an entry inside its class
    int* ccount = (int*)(smem + LDS_TOTAL - 256);     // [16] entries per class
    {
      // wave w numbers the entries of classes w + 1 and w + 9
      const unsigned ma = (unsigned)wave + 1u, mb = (unsigned)wave + 9u;   // mb = 16 for the last wave: no such class
      int ca = 0, cb = 0;
      for (int base = 0; base < nR; base += 64) {
        const int i = base + lane;
        const unsigned m4 = i < nR ? rest[i] >> 28 : 0u;
        const unsigned long long ba = __ballot(m4 == ma), bb = __ballot(m4 == mb);
        if (m4 == ma) upos[i] = (unsigned)(ca + lanes_before(ba));
        if (m4 == mb) upos[i] = (unsigned)(cb + lanes_before(bb));
        ca += __popcll(ba);
        cb += __popcll(bb);
      }
      if (lane == 0) {
        ccount[ma] = ca;
        if (mb < 16u) ccount[mb] = cb;
        if (wave == 0) ccount[0] = 0;
      }
    }
    __syncthreads();
    unsigned* sorted = upos + union_max;
    for (int i = threadIdx.x; i < nR; i += 512) {
      const unsigned e = rest[i];
      const int m = (int)(e >> 28);
      const int c = ccount[m];
      const int a2 = 2 * (int)upos[i] + 1;            // my key is a2 / (2c)
      const float rc = 1.0f / (float)c;
      int rank = 0;
#pragma unroll
      for (int m2 = 1; m2 < 16; ++m2) {
        const int c2 = ccount[m2];
        if (c2 == 0) continue;
        // entries j of class m2 with (2j+1)/(2 c2) < a2/(2c), i.e. (2j+1) c < a2 c2
        const int A = a2 * c2;                        // below 2^24 (the lists fit in LDS): exact in float
        int fl = (int)((float)A * rc);                // floor(A / c) up to one unit, put right below
        int rem = A - fl * c;
        if (rem < 0) {
          fl -= 1;
          rem += c;
        } else if (rem >= c) {
          fl += 1;
          rem -= c;
        }
        int cntl = (fl + (rem != 0)) >> 1;            // ceil(A / c) / 2
        // an exact tie goes to the lower class number
        if (m2 < m && rem == 0 && (fl & 1)) cntl += 1;
        rank += min(cntl, c2);
      }
      sorted[rank] = e;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nR; i += 512) rest[i] = sorted[i];
    __syncthreads();
  }

  // ---- per-lane constants
  const int r = lane & 31, hh = lane >> 5;
  const int krow = sigma(r);
  const int ke = (hh ^ (krow & 15)) << 4;
  int kofs[8];                                        // K operand offsets inside a slot, swizzle applied
#pragma unroll
  for (int t = 0; t < 8; ++t) kofs[t] = krow * 256 + ((32 * t) ^ ke);
  const unsigned ring_lds = (unsigned)(uintptr_t)(lds_bytes)smem;
  unsigned koff[4];
  tile_lane_offsets<256>(lane, koff);
  const unsigned char* Kbh = Kp + bh * q.n_pad * (D * 2);
  const unsigned char* Vlane = Vt + bh * q.n_pad * (D * 2) + lane * 16;
  // one wave brings the K tile of union entry u into ring slot u % RING
  const int live_waves = __builtin_amdgcn_readfirstlane(ctrl[28]);
  auto issue_tile = [&](int u) {
    const unsigned e = (unsigned)__builtin_amdgcn_readfirstlane((int)ulist[u]);
    // how many waves will read the tile: the live waves of the query blocks that hold the entry
    int readers = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const int qb_w = SUB == 1 ? (w + 2 * (w >> 2)) & 3 : w >> 2;
      readers += (live_waves >> w) & (int)(e >> (28 + qb_w)) & 1;
    }
    if (lane == 0) __atomic_store_n(&left[u & (RING - 1)], readers, __ATOMIC_RELAXED);   // (before the transfer, hence before the slot is published)
    const long long j = (long long)(e & 0x3fffffu);
    dma_tile(Kbh + j * K_TILE, ring_lds + (unsigned)(u & (RING - 1)) * SLOT, koff);
  };
  int pending = -1;
  // a tile this wave has requested becomes visible to the others once it has landed
  auto publish = [&]() {
    const int pd = __builtin_amdgcn_readfirstlane(pending);   // (the same in every lane; says so to the compiler)
    if (pd >= 0) {
      wait_vm0();
      if (lane == 0) __atomic_store_n(&ready[pd & (RING - 1)], pd, __ATOMIC_RELAXED);
      pending = -1;
    }
  };

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  Soft st;
  st.m = -INFINITY;
  st.top = -INFINITY;
  st.l = 0.f;
  // Make the compiler wait for the Q fragments here, by touching them: its own counter
  // bookkeeping then knows they are in.  Otherwise it would wait for them at their first use
  // inside the tile loop, with a vmcnt that also drains the tile loads in flight.
#pragma unroll
  for (int t = 0; t < 8; ++t) asm volatile("" : "+v"(qf[t]));

  const unsigned my_bit = live ? (1u << (28 + qblk)) : 0u;
  const bool pad_query = 32 * part + r >= valid_slots(q, per_frame, pos);
  // a look at the whole control block: lane i holds ctrl[i]
  auto look = [&]() -> int { return __atomic_load_n(ctrl + (lane & 31), __ATOMIC_RELAXED); };
  // request the next tile if the ring has room, judging by a look c (which may be old: then the
  // compare-and-swap fails or the room is underestimated, both harmless)
  auto service = [&](int c) {
    if (__builtin_amdgcn_readfirstlane(pending) >= 0) return;   // at most one request of mine in flight
    const int L = __builtin_amdgcn_readlane(c, 16);
    if (L >= nU) return;
    // its slot is free once every reader of the entry it holds has left it (and that entry did arrive)
    const int sl = L & (RING - 1);
    if (__builtin_amdgcn_readlane(c, 8 + sl) != 0) return;
    if (L >= RING && __builtin_amdgcn_readlane(c, sl) != L - RING) return;
    int got = L + 1;
    if (lane == 0) got = atomicCAS(next_load, L, L + 1);
    got = __builtin_amdgcn_readfirstlane(got);
    if (got != L) return;
    issue_tile(L);
    pending = L;
  };
  bool gave_up = false;
  int tiles_seen = 0, tiles_kept = 0;                 // (scalar registers; reported when the caller asks for the counts)
  int snap = look();
  // The walk, 64 entries at a time: lane i holds entry base + i, a ballot tells which of them
  // are mine.  Entries that are not mine cost nothing.
  for (int base = 0; base < nU && !gave_up; base += 64) {
    const unsigned e_lane = base + lane < nU ? ulist[base + lane] : 0u;
    unsigned long long mine = __ballot((e_lane & my_bit) != 0u);
    while (mine) {
      const int i = (int)__builtin_ctzll(mine);
      mine &= mine - 1;
      const int u = base + i;
      const int slot_i = u & (RING - 1);
      publish();                                      // my last request has had a whole tile's time to land
      if (__builtin_amdgcn_readlane(snap, slot_i) != u) {
        int spins = 0;
        for (;;) {
          snap = look();
          service(snap);
          if (__builtin_amdgcn_readlane(snap, slot_i) == u) break;
          if (__builtin_amdgcn_readfirstlane(pending) >= 0) {
            publish();                                // idle anyway: wait for my own request and hand it over
          } else {
            __builtin_amdgcn_s_sleep(1);
            if (++spins > kSpinLimit) {
              gave_up = true;
              break;
            }
          }
        }
        if (gave_up) break;
      }
      const int fresh = look();                       // asked for now, used after the tile: its latency hides behind the tile
      const unsigned e = (unsigned)__builtin_amdgcn_readlane((int)e_lane, i);
      {
        const int nv = (int)((e >> 22) & 63u) + 1;
        const unsigned char* slot = smem + slot_i * SLOT;
        const unsigned char* kaddr[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) kaddr[t] = slot + kofs[t];
        const bool kept = compute_tile(kaddr, Vlane + (long long)(e & 0x3fffffu) * V_TILE, hh, nv, pad_query, skip, qf, o, st);
        tiles_seen += 1;
        tiles_kept += kept ? 1 : 0;
      }
      // my reads of the slot are complete: one reader less
      wait_lds();
      if (lane == 0) atomicSub(&left[slot_i], 1);
      // (Only waves that are waiting for a tile ask for tiles: having every wave look for room after each of
      // its tiles cost the busy ones more than the earlier requests saved.)
      snap = fresh;
    }
  }
  publish();
  if (tile_counts != nullptr && lane == 0 && tiles_seen) {
    atomicAdd(&tile_counts[0], (unsigned long long)tiles_seen);
    atomicAdd(&tile_counts[1], (unsigned long long)tiles_kept);
  }
  if (gave_up && lane == 0) atomicAdd(&g_wait_failures, 1ull);
  __syncthreads();                                    // everyone is done with the ring: reuse it to stage the output
  if (!live) {
    // 32 pad slots and nothing else: their rows of the reordered output are zeroed (in the original
    // order they do not exist)
    if (has_block && !direct) {
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row = it * 4 + (lane >> 4), ch = lane & 15;
        *(uint4*)(Op + (qb * BLOCK + 32 * part + row) * (D * 2) + ch * 16) = make_uint4(0u, 0u, 0u, 0u);
      }
      if (lse && lane < 32) lse[qb * BLOCK + 32 * part + lane] = 0.f;
    }
    return;
  }

  // ---- epilogue: normalise, convert, stage through LDS, write rows of 256 B
  unsigned char* stage = smem + wave * (RING_BYTES / WAVES);
  {
    const float lt = sum_across_halves(st.l);
    const float inv = lt > 0.f ? 1.0f / lt : 0.f;     // 0 only in pad query slots whose wave skipped every tile
    if (lse && hh == 0) lse[qb * BLOCK + 32 * part + r] = st.m * kScale + __logf(lt);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        // registers 4a..4a+3 are d = 32dt + 8a + 4hh + 0..3 of query r
        f32x2 v0 = {o[dt][4 * a] * inv, o[dt][4 * a + 1] * inv};
        f32x2 v1 = {o[dt][4 * a + 2] * inv, o[dt][4 * a + 3] * inv};
        bf16x2 b0 = __builtin_convertvector(v0, bf16x2);
        bf16x2 b1 = __builtin_convertvector(v1, bf16x2);
        uint2 w2 = make_uint2(*(unsigned*)&b0, *(unsigned*)&b1);
        if (gave_up) w2 = make_uint2(0x7fc07fc0u, 0x7fc07fc0u);   // a wait ran out: say so with NaN rather than with wrong numbers
        *(uint2*)(stage + r * O_STRIDE + (32 * dt + 8 * a + 4 * hh) * 2) = w2;
      }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 4 + (lane >> 4), ch = lane & 15;
    const long long orow = row_bytes(32 * part + row, q.out);
    if (orow >= 0) *(uint4*)(Op + orow + ch * 16) = *(const uint4*)(stage + row * O_STRIDE + ch * 16);
  }
}

}  // namespace ring

// LDS left beside the ring: four bitmaps of g bits, the union list (at most min(g, 4k) entries)
// and, for the balanced walk, two more arrays of that length.
// 0: the kernel cannot run this problem; 1: it can, walking in ascending order; 2: balanced walk.
int attn_bf16_ring_fits(const Geo& q, bool any_length) {
  if (q.block != ring::BS && q.block != 2 * ring::BS) return 0;
  const int sub = q.block / ring::BS, fg = 4 / sub;
  if ((long long)q.g * sub >= (1 << 22)) return 0;
  long long union_max = sub * ((long long)q.g < (long long)fg * q.k || any_length ? q.g : (long long)fg * q.k);
  long long base = 4LL * 4 * ((q.g + 31) / 32) + 4 * union_max + 512;
  if (base > ring::AUX_BYTES) return 0;
  return base + 8 * union_max <= ring::AUX_BYTES ? 2 : 1;
}

hipError_t launch_attn_bf16_ring(const Geo& q, const void* Qp, const void* Kp, const void* Vt, const int32_t* idx,
                                 const int32_t* row_ptr, long long cap, void* Op, float* lse, bool direct,
                                 unsigned long long* tile_counts, hipStream_t s) {
  const int per_frame = q.gh * q.gw;
  const int sub = q.block / ring::BS, fg = 4 / sub;
  const ring::TailPlan plan = ring::tail_plan(q, fg);
  unsigned grid = (unsigned)((long long)q.B * q.H * (8 * ((per_frame + 7) / 8) * plan.full_groups + plan.tail_wgs));
  const int balance = attn_bf16_ring_fits(q, row_ptr != nullptr) == 2 ? 1 : 0;
  const float skip = log2f((float)q.k * (float)q.block) + ring::kDropLog2;
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(512), 0, s, q, (const unsigned char*)Qp, (const unsigned char*)Kp,
                       (const unsigned char*)Vt, idx, row_ptr, cap, (unsigned char*)Op, lse, balance, skip, direct ? 1 : 0, tile_counts);
  };
  if (sub == 1 && !row_ptr) go(ring::attn_bf16_ring_kernel<1, false>);
  else if (sub == 1) go(ring::attn_bf16_ring_kernel<1, true>);
  else if (!row_ptr) go(ring::attn_bf16_ring_kernel<2, false>);
  else go(ring::attn_bf16_ring_kernel<2, true>);
  return hipGetLastError();
}

// Waves that gave up waiting for a tile since the library was loaded on the current device (synchronises).
hipError_t read_wait_failures(unsigned long long* count) {
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) return e;
  return hipMemcpyFromSymbol(count, HIP_SYMBOL(ring::g_wait_failures), sizeof(*count), 0, hipMemcpyDeviceToHost);
}

}  // namespace da
