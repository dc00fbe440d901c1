// Reordering by pi (Algorithm 1) and restoring by pi^-1 (Algorithm 2) as pure data movement.
// HBM-bound: every element is read once and written once in 16-byte pieces; the index
// arithmetic is done on the fly, no index array is read.
#include "da_internal.h"

namespace da {

typedef uint4 chunk16;  // 16 bytes

// a source chunk is read exactly once by these kernels: non-temporal, so that the stream leaves the L2 to others
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ inline chunk16 load_once(const chunk16* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// perm / inv / valid arrays for callers that want them.
__global__ void build_perm_kernel(Geo q, int32_t* perm, int32_t* inv, int32_t* valid) {
  long long slot = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (slot >= q.n_pad) return;
  int i = (int)(slot / q.block);
  int s = (int)(slot - (long long)i * q.block);
  BlockPos b = block_pos(q, i);
  int nv = b.vh * b.vw;
  int tok = -1;
  if (s < nv) {
    int u = s / b.vw, v = s - u * b.vw;
    tok = (b.f * q.fh + b.y0 + u) * q.fw + b.x0 + v;
    if (inv) inv[tok] = (int32_t)slot;
  }
  if (perm) perm[slot] = tok;
  if (valid && s == 0) valid[i] = nv;
}

// One workgroup per (block, batch*head).  cpr = 16-byte chunks per row.
// FWD: Y[slot] = X[pi[slot]] or zeros;  !FWD: X-order output, Y[token] = Xp[slot].
// The reordered side is contiguous [B,H,n_pad,d]; the other side is the caller's tensor (q.in for
// the source of FWD, q.out for the destination of !FWD).
template <bool FWD>
__global__ __launch_bounds__(256) void permute_rows_kernel(Geo q, const chunk16* __restrict__ X, chunk16* __restrict__ Y,
                                                            int cpr) {
  int i = blockIdx.x;
  long long bh = blockIdx.y;
  BlockPos b = block_pos(q, i);
  int nv = b.vh * b.vw;
  const int per = q.d / cpr;                           // elements per chunk
  const Rows& far = FWD ? q.in : q.out;
  const long long far0 = row_offset(far, q.H, bh, block_first_row(q, i, b)) / per;   // chunk of the block's first row
  const long long far_sn = far.sn / per, pitch = block_row_pitch(q, b);
  const long long near0 = (bh * q.n_pad + (long long)i * q.block) * cpr;
  int total = (FWD ? q.block : nv) * cpr;
  for (int e = threadIdx.x; e < total; e += blockDim.x) {
    int s = e / cpr, c = e - s * cpr;
    if (FWD) {
      chunk16 val = make_uint4(0, 0, 0, 0);
      if (s < nv) {
        int u = s / b.vw, v = s - u * b.vw;
        val = load_once(&X[far0 + ((long long)u * pitch + v) * far_sn + c]);
      }
      Y[near0 + (long long)s * cpr + c] = val;
    } else {
      int u = s / b.vw, v = s - u * b.vw;
      Y[far0 + ((long long)u * pitch + v) * far_sn + c] = load_once(&X[near0 + (long long)s * cpr + c]);
    }
  }
}

// Block-transposed reorder: Xt[bh][i][c][s] = X[bh][pi[i*block+s]][c] (zeros in pad slots).
// One workgroup per (block, batch*head).  The block's rows go through LDS; ES = element bytes.
// OPERAND (bf16, block a multiple of 64, d a multiple of 32): the same transposed block, written as
// the 16-byte operands of the matrix instructions, one 64-slot sub-block after the other: unit
// ((t*nd + dt)*64 + hh*32 + r) of sub-block sb holds channel 32dt + r, slots 64sb + 16t + 8hh + 0..7.
template <typename E, bool OPERAND>
__global__ __launch_bounds__(256) void permute_vt_kernel(Geo q, const E* __restrict__ X, E* __restrict__ Y) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int PER = 16 / sizeof(E);  // elements per 16-byte chunk
  E* tile = (E*)smem;                  // [block][d + PER] (padded rows)
  const int ld = q.d + PER;
  int i = blockIdx.x;
  long long bh = blockIdx.y;
  BlockPos b = block_pos(q, i);
  int nv = b.vh * b.vw;
  int cpr = q.d / PER;
  const chunk16* Xc = (const chunk16*)(X + row_offset(q.in, q.H, bh, block_first_row(q, i, b)));   // the block's first row
  const long long sn = q.in.sn / PER, pitch = block_row_pitch(q, b);
  for (int e = threadIdx.x; e < q.block * cpr; e += blockDim.x) {
    int s = e / cpr, c = e - s * cpr;
    chunk16 val = make_uint4(0, 0, 0, 0);
    if (s < nv) {
      int u = s / b.vw, v = s - u * b.vw;
      val = load_once(&Xc[((long long)u * pitch + v) * sn + c]);
    }
    *(chunk16*)(tile + s * ld + c * PER) = val;
  }
  __syncthreads();
  E* out = Y + (bh * q.g + i) * (long long)q.d * q.block;
  if (OPERAND) {
    const int nd = q.d >> 5, per_half = q.d * 64 / PER;   // 16-byte units per 64-slot sub-block
    for (int e = threadIdx.x; e < q.d * q.block / PER; e += blockDim.x) {
      const int sb = e / per_half, eh = e - sb * per_half;
      const int r = eh & 31, hh = (eh >> 5) & 1, grp = eh >> 6;
      const int t = grp / nd, dt = grp - t * nd;
      const int c = 32 * dt + r, s0 = 64 * sb + 16 * t + 8 * hh;
      E tmp[PER];
#pragma unroll
      for (int j = 0; j < PER; ++j) tmp[j] = tile[(s0 + j) * ld + c];
      *(chunk16*)(out + (long long)e * PER) = *(chunk16*)tmp;
    }
    return;
  }
  int spr = q.block / PER;  // 16-byte chunks per output row (a row holds `block` slots of one channel)
  for (int e = threadIdx.x; e < q.d * spr; e += blockDim.x) {
    int c = e / spr, s8 = e - c * spr;
    E tmp[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) tmp[j] = tile[(s8 * PER + j) * ld + c];
    *(chunk16*)(out + (long long)c * q.block + s8 * PER) = *(chunk16*)tmp;
  }
}

hipError_t launch_build_perm(const Geo& q, int32_t* perm, int32_t* inv, int32_t* valid, hipStream_t s) {
  unsigned blocks = (unsigned)((q.n_pad + 255) / 256);
  hipLaunchKernelGGL(build_perm_kernel, dim3(blocks), dim3(256), 0, s, q, perm, inv, valid);
  return hipGetLastError();
}

hipError_t launch_permute(const Geo& q, const void* X, void* Y, int mode, hipStream_t s) {
  size_t es = q.dtype == DA_BF16 ? 2 : 4;
  int cpr = (int)(q.d * es / 16);
  dim3 grid((unsigned)q.g, (unsigned)(q.B * q.H));
  if (mode == DA_REORDER_ROWS) {
    hipLaunchKernelGGL(permute_rows_kernel<true>, grid, dim3(256), 0, s, q, (const chunk16*)X, (chunk16*)Y, cpr);
  } else if (mode == DA_RESTORE) {
    hipLaunchKernelGGL(permute_rows_kernel<false>, grid, dim3(256), 0, s, q, (const chunk16*)X, (chunk16*)Y, cpr);
  } else {
    size_t per = 16 / es;
    size_t lds = (size_t)q.block * (q.d + per) * es;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    if (mode == DA_REORDER_VOP)
      hipLaunchKernelGGL((permute_vt_kernel<uint16_t, true>), grid, dim3(256), lds, s, q, (const uint16_t*)X, (uint16_t*)Y);
    else if (es == 2)
      hipLaunchKernelGGL((permute_vt_kernel<uint16_t, false>), grid, dim3(256), lds, s, q, (const uint16_t*)X, (uint16_t*)Y);
    else
      hipLaunchKernelGGL((permute_vt_kernel<uint32_t, false>), grid, dim3(256), lds, s, q, (const uint32_t*)X, (uint32_t*)Y);
  }
  return hipGetLastError();
}

}  // namespace da
