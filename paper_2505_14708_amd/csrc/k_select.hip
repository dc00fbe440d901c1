// Guided sparsity: per row of the draft scores keep the k largest entries (ties to the
// lowest column) and emit their columns in ascending order.
//
// One wavefront per row.  The row is mapped to order-preserving 32-bit keys; the value of the
// k-th largest key is found bit by bit from the top (32 counting passes); one more ordered pass
// writes every column whose key beats the threshold plus the first (k - #greater) columns that
// equal it, using ballot + lane-prefix popcounts so the output stays in column order without
// any sort.  Rows of up to 4096 columns are held in registers (lane l keeps columns l, l + 64,
// ...): a counting pass is then one compare per key, whose lane mask is counted on the scalar
// unit.  Longer rows keep their keys in LDS, or recompute them from global memory.
#include "da_internal.h"

namespace da {

__device__ inline unsigned order_key(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;       // NaN ranks below everything
  if ((u & 0x7fffffffu) == 0u) u = 0u;                  // -0 == +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline int wave_sum_int(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// number of set bits of `m` strictly below this lane
__device__ inline int lane_prefix(unsigned long long m) {
  return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0));
}

template <bool IN_LDS>
__global__ __launch_bounds__(64) void select_kernel(const float* __restrict__ scores, int32_t* __restrict__ idx,
                                                    uint8_t* __restrict__ mask, int g, int k) {
  extern __shared__ unsigned lds_keys[];
  const long long row = blockIdx.x;
  const int lane = threadIdx.x;
  const float* in = scores + row * g;
  // without room in LDS the keys are recomputed from global memory in every pass
  auto key_at = [&](int j) -> unsigned { return IN_LDS ? lds_keys[j] : order_key(in[j]); };
  if (IN_LDS) {
    for (int j = lane; j < g; j += 64) lds_keys[j] = order_key(in[j]);
    __syncthreads();
  }
  unsigned thr = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    unsigned cand = thr | (1u << bit);
    int cnt = 0;
    for (int j = lane; j < g; j += 64) cnt += key_at(j) >= cand ? 1 : 0;
    cnt = wave_sum_int(cnt);
    if (cnt >= k) thr = cand;
  }
  // thr is now the k-th largest key
  int gt = 0;
  for (int j = lane; j < g; j += 64) gt += key_at(j) > thr ? 1 : 0;
  gt = wave_sum_int(gt);
  int need_eq = k - gt;
  int written = 0, eq_seen = 0;
  int32_t* out = idx + row * k;
  uint8_t* mrow = mask ? mask + row * g : nullptr;
  for (int j0 = 0; j0 < g; j0 += 64) {
    int j = j0 + lane;
    unsigned key = j < g ? key_at(j) : 0u;
    bool is_gt = j < g && key > thr;
    bool is_eq = j < g && key == thr;
    unsigned long long eq_mask = __ballot(is_eq);
    bool take = is_gt || (is_eq && eq_seen + lane_prefix(eq_mask) < need_eq);
    unsigned long long take_mask = __ballot(take);
    if (take) out[written + lane_prefix(take_mask)] = j;
    if (mrow && j < g) mrow[j] = take ? 1 : 0;
    written += __popcll(take_mask);
    eq_seen += __popcll(eq_mask);
  }
}


// Keys in registers: KPL keys per lane, column of key i of lane l is l + 64 i.
// READ_ON: a column past the end of the row may be read from the rows that follow (the launcher gives this
// instantiation only rows for which that stays inside the array).
template <int KPL, bool READ_ON>
__global__ __launch_bounds__(64, KPL == 64 ? 4 : 1) void select_reg_kernel(const float* __restrict__ scores, int32_t* __restrict__ idx,
                                                        uint8_t* __restrict__ mask, int g, int k) {
  const long long row = blockIdx.x;
  const int lane = threadIdx.x;
  const float* in = scores + row * g;
  unsigned key[KPL];
  {
    // Every load of the row is asked for before the first is used, none behind a branch of its own.  A column past
    // the end of the row reads on into the rows that follow (what it reads is not used): the addresses are then one
    // base plus constants, two registers instead of two per load, and twice as many rows fit a SIMD.  The rows so
    // close to the end of the array that this would leave it read their last column instead.
    float x[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) x[i] = READ_ON ? in[lane + 64 * i] : in[min(lane + 64 * i, g - 1)];
#pragma unroll
    for (int i = 0; i < KPL; ++i)
      key[i] = lane + 64 * i < g ? order_key(x[i]) : 0u;   // a column past the end never counts: every trial value is > 0
  }
  unsigned thr = 0u;
  bool cut = false;                                   // exactly k keys are >= thr: no tie to resolve, no bit left to find
  for (int bit = 31; bit >= 0; --bit) {
    const unsigned cand = thr | (1u << bit);
    int cnt = 0;
    // (eight keys at a time: with all the lane masks of a pass alive at once the scalar registers run out)
#pragma unroll
    for (int i0 = 0; i0 < KPL; i0 += 8) {
#pragma unroll
      for (int i = i0; i < i0 + 8; ++i) cnt += __popcll(__ballot(key[i] >= cand));
      __builtin_amdgcn_sched_barrier(0);
    }
    if (cnt >= k) thr = cand;
    if (cnt == k) {                                   // (the same in every lane)
      cut = true;
      break;
    }
  }
  // thr is now the k-th largest key, or (cut) a value that exactly k keys reach
  int gt = 0;
  if (cut) {
    gt = k;                                           // all of them count as "greater": take key >= thr below
    thr -= 1u;                                        // thr >= 1 here: a trial value is never 0
  } else {
#pragma unroll
    for (int i = 0; i < KPL; ++i) gt += __popcll(__ballot(key[i] > thr));
  }
  const int need_eq = k - gt;
  int written = 0, eq_seen = 0;
  int32_t* out = idx + row * k;
  uint8_t* mrow = mask ? mask + row * g : nullptr;
#pragma unroll
  for (int i = 0; i < KPL; ++i) {
    const int j = lane + 64 * i;
    if (64 * i >= g) break;                           // uniform
    const bool is_gt = j < g && key[i] > thr;
    const bool is_eq = j < g && key[i] == thr;
    const unsigned long long eq_mask = __ballot(is_eq);
    const bool take = is_gt || (is_eq && eq_seen + lane_prefix(eq_mask) < need_eq);
    const unsigned long long take_mask = __ballot(take);
    if (take) out[written + lane_prefix(take_mask)] = j;
    if (mrow && j < g) mrow[j] = take ? 1 : 0;
    written += __popcll(take_mask);
    eq_seen += __popcll(eq_mask);
  }
}

// Every block kept (k = g, or a whole-map budget of g*g entries): the lists are 0 .. g-1 whatever the scores are.
// idx: per head g rows of g columns, heads `head_stride` entries apart; row_ptr (optional): [B*H, g+1] offsets i*g.
__global__ __launch_bounds__(256) void all_lists_kernel(int32_t* __restrict__ idx, int32_t* __restrict__ row_ptr, int g,
                                                        long long head_stride) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long bh = blockIdx.y;
  if (e < (long long)g * g) idx[bh * head_stride + e] = (int32_t)(e % g);
  if (row_ptr && e <= g) row_ptr[bh * (g + 1) + e] = (int32_t)(e * g);
}

hipError_t launch_all_lists(const Geo& q, int32_t* idx, int32_t* row_ptr, long long head_stride, hipStream_t s) {
  const long long per_head = (long long)q.g * q.g;
  dim3 grid((unsigned)((per_head + 256) / 256), (unsigned)(q.B * q.H));   // (+256: entry g*g itself is row_ptr's last)
  hipLaunchKernelGGL(all_lists_kernel, grid, dim3(256), 0, s, idx, row_ptr, q.g, head_stride);
  return hipGetLastError();
}

template <int KPL>
static void launch_select_reg(const Geo& q, long long rows, const float* scores, int32_t* idx, uint8_t* mask, bool slack,
                              hipStream_t s) {
  // rows whose 64 * KPL columns starting at the row's first all lie inside the array: all but the last few, or all
  // of them when the caller vouches for kSelectSlack readable bytes behind the array
  const long long spill = 64LL * KPL - q.g;           // columns read past the end of a row (>= 0)
  const long long last = spill > 0 && !slack ? (spill + q.g - 1) / q.g : 0;
  const long long head = rows > last ? rows - last : 0;
  if (head > 0)
    hipLaunchKernelGGL((select_reg_kernel<KPL, true>), dim3((unsigned)head), dim3(64), 0, s, scores, idx, mask, q.g, q.k);
  if (rows > head)
    hipLaunchKernelGGL((select_reg_kernel<KPL, false>), dim3((unsigned)(rows - head)), dim3(64), 0, s, scores + head * q.g,
                       idx + head * q.k, mask ? mask + head * q.g : nullptr, q.g, q.k);
}

hipError_t launch_select(const Geo& q, const float* scores, int32_t* idx, uint8_t* mask, bool slack, hipStream_t s) {
  long long rows = (long long)q.B * q.H * q.g;
  size_t lds = (size_t)q.g * sizeof(unsigned);
  if (q.g <= 64 * 16)
    launch_select_reg<16>(q, rows, scores, idx, mask, slack, s);
  else if (q.g <= 64 * 32)
    launch_select_reg<32>(q, rows, scores, idx, mask, slack, s);
  else if (q.g <= 64 * 64)
    launch_select_reg<64>(q, rows, scores, idx, mask, slack, s);
  else if (lds <= 64 * 1024)
    hipLaunchKernelGGL(select_kernel<true>, dim3((unsigned)rows), dim3(64), lds, s, scores, idx, mask, q.g, q.k);
  else
    hipLaunchKernelGGL(select_kernel<false>, dim3((unsigned)rows), dim3(64), 0, s, scores, idx, mask, q.g, q.k);
  return hipGetLastError();
}

}  // namespace da
