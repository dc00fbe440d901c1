// Internal declarations shared by the host API and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "da.h"

namespace da {

// Where the rows of a [B, H, rows, d] tensor of the caller live: offsets in elements between consecutive
// batches, heads and rows (a row of d elements is contiguous).
struct Rows {
  long long sb, sh, sn;
};

// Everything the kernels need to know about one problem (passed by value).
struct Geo {
  int B, H, T, fh, fw, d;
  int ph, pw, gh, gw;
  int g, block, k;
  int dtype;
  int pool;          // DA_POOL_AVG / DA_POOL_MAX
  long long n, n_pad;
  // The caller's Q, K, V (in) and O (out).  reordered == 0: rows are tokens in the original order
  // (n per head); 1: rows are the slots of Algorithm 1's order (n_pad per head, pad rows zero).
  Rows in, out;
  int reordered;
};

// element offset of row `row` of (batch, head) number bh
__host__ __device__ inline long long row_offset(const Rows& r, int H, long long bh, long long row) {
  const long long b = bh / H, h = bh - b * H;
  return b * r.sb + h * r.sh + row * r.sn;
}

// Block i (in Algorithm 1's frame / patch-row / patch-column order) -> its frame, the
// token coordinates of its top-left corner and its valid extent.
struct BlockPos {
  int f, y0, x0, vh, vw;
};

__host__ __device__ inline BlockPos block_pos(const Geo& q, int i) {
  BlockPos b;
  int per_frame = q.gh * q.gw;
  b.f = i / per_frame;
  int r = i - b.f * per_frame;
  int bi = r / q.gw;
  int bj = r - bi * q.gw;
  b.y0 = bi * q.ph;
  b.x0 = bj * q.pw;
  b.vh = min(q.ph, q.fh - b.y0);
  b.vw = min(q.pw, q.fw - b.x0);
  return b;
}

__host__ __device__ inline int block_valid(const Geo& q, int i) {
  BlockPos b = block_pos(q, i);
  return b.vh * b.vw;
}

// First row of block i in the caller's Q, K, V, O (slot 0 of the block) and the distance in rows between the
// block's patch rows: slot s = u * vw + v of the block is row first + u * pitch + v.
__host__ __device__ inline long long block_first_row(const Geo& q, int i, const BlockPos& b) {
  return q.reordered ? (long long)i * q.block : ((long long)b.f * q.fh + b.y0) * q.fw + b.x0;
}
__host__ __device__ inline int block_row_pitch(const Geo& q, const BlockPos& b) { return q.reordered ? b.vw : q.fw; }

// Original token index -> slot in the reordered sequence (pi^-1 of Algorithm 2).
__host__ __device__ inline long long token_slot(const Geo& q, long long n) {
  int per = q.fh * q.fw;
  int f = (int)(n / per);
  int r = (int)(n - (long long)f * per);
  int y = r / q.fw, x = r - y * q.fw;
  int bi = y / q.ph, u = y - bi * q.ph;
  int bj = x / q.pw, v = x - bj * q.pw;
  int vw = min(q.pw, q.fw - bj * q.pw);
  long long blk = ((long long)f * q.gh + bi) * q.gw + bj;
  return blk * q.block + u * vw + v;
}

// launchers (each returns hipGetLastError() after its launches)
hipError_t launch_build_perm(const Geo& q, int32_t* perm, int32_t* inv, int32_t* valid, hipStream_t s);
hipError_t launch_permute(const Geo& q, const void* X, void* Y, int mode, hipStream_t s);
hipError_t launch_pool(const Geo& q, const void* Q, const void* K, float* q_pool, float* k_pool, hipStream_t s);
// pooling and the reordering of Q and K (DA_REORDER_ROWS layout) in one pass over Q and K
hipError_t launch_pool_reorder(const Geo& q, const void* Q, const void* K, float* q_pool, float* k_pool, void* Qp,
                               void* Kp, hipStream_t s);
hipError_t launch_draft_logits(const Geo& q, const float* q_pool, const float* k_pool, float* logits, hipStream_t s);
hipError_t launch_row_softmax(const Geo& q, const float* logits, float* draft, hipStream_t s);
// slack: kSelectSlack bytes behind `scores` may be read (their values are not used); without it the last few rows go
// through a second launch that stays inside the array
constexpr size_t kSelectSlack = 64 * 64 * sizeof(float);
hipError_t launch_select(const Geo& q, const float* scores, int32_t* idx, uint8_t* mask, bool slack, hipStream_t s);
hipError_t launch_all_lists(const Geo& q, int32_t* idx, int32_t* row_ptr, long long head_stride, hipStream_t s);
// idx: k columns per row; or, with row_ptr [B,H,g+1], lists of any length, the lists of head bh one after the
// other from idx + bh * cap on
hipError_t launch_attn_f32(const Geo& q, const float* Qp, const float* Kp, const float* Vt, const int32_t* idx,
                           const int32_t* row_ptr, long long cap, float* Op, float* lse, hipStream_t s);
// whole-map threshold selection (k_select_global.hip)
size_t select_global_workspace(const Geo& q);
// device address, on the current device, of the library's built-in scratch (DA_STATIC_SCRATCH_BYTES bytes)
hipError_t static_scratch(void** ptr);
hipError_t launch_select_global(const Geo& q, long long budget, long long cap, const float* scores, int32_t* row_ptr,
                                int32_t* cols, uint8_t* mask, void* ws, hipStream_t s);
// bf16 block-sparse attention (k_attn_bf16_ring.hip)
int attn_bf16_ring_fits(const Geo& q, bool any_length = false);
// direct: Qp and Op are Q and O in the original token order (lse stays in slot order)
// tile_counts (may be NULL): two counters the waves add to: tiles gone through, tiles whose second product ran
hipError_t launch_attn_bf16_ring(const Geo& q, const void* Qp, const void* Kp, const void* Vt, const int32_t* idx,
                                 const int32_t* row_ptr, long long cap, void* Op, float* lse, bool direct,
                                 unsigned long long* tile_counts, hipStream_t s);
hipError_t read_wait_failures(unsigned long long* count);

}  // namespace da
