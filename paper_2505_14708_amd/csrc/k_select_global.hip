// Guided sparsity in its whole-map form (Section 3.2.2, "Error from Sparsity Mask"): the threshold t is
// the ceil(r g^2)-th largest score of a head's g x g map and M_ij = 1 for the scores that reach it.
//
// Per head: the scores are mapped to order-preserving 32-bit keys and the key of rank `budget` is found
// by a radix select from the top (digits of 11, 11 and 10 bits): a pass builds the histogram of the next
// digit over the keys that agree with the digits found so far, a small kernel walks the histogram from
// the top and fixes the digit.  Then every row counts its keys above and at the threshold, one workgroup
// per head turns the counts into the row offsets (keys equal to the threshold are taken in row-major order
// until the budget is used up; a row left empty keeps its best column), and every row writes its kept
// columns in ascending order with an ordered ballot compaction.  Exact and deterministic.
#include "da_internal.h"

namespace da {
namespace {

constexpr int kBins = 2048;
constexpr int kHistThreads = 256;
constexpr int kKeysPerThread = 16;                    // keys a thread of the histogram pass takes
constexpr int kChunk = kHistThreads * kKeysPerThread;
constexpr int kChunksPerGroup = 8;                    // chunks a workgroup takes before it adds its counts to the head's

__device__ inline unsigned gkey(float x) {
  unsigned u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;     // NaN ranks below everything
  if ((u & 0x7fffffffu) == 0u) u = 0u;                // -0 == +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline int lanes_below(unsigned long long m) {
  return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0));
}

// per-head state of the search: the high bits found so far and the rank still looked for among the
// keys that carry them
struct SelState {
  unsigned prefix;
  unsigned rank;
};

// digit of pass p of a key, and the bits above it
__device__ inline unsigned digit_of(unsigned key, int pass) {
  return pass == 0 ? key >> 21 : pass == 1 ? (key >> 10) & 2047u : key & 1023u;
}
__device__ inline unsigned above_of(unsigned key, int pass) { return pass == 0 ? 0u : pass == 1 ? key >> 21 : key >> 10; }

__global__ void zero_words_kernel(unsigned* p, long long n) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// hist[bh][pass][bin] += number of keys of head bh whose higher digits equal the state's prefix and whose
// digit of this pass is `bin`.  One workgroup takes kChunk consecutive scores of one head.
template <int PASS>
__global__ __launch_bounds__(kHistThreads) void hist_kernel(const float* __restrict__ scores, unsigned* __restrict__ hist,
                                                           const SelState* __restrict__ state, long long g2) {
  constexpr int pass = PASS;
  __shared__ unsigned lh[kBins];
  const long long bh = blockIdx.y;
  for (int i = threadIdx.x; i < kBins; i += kHistThreads) lh[i] = 0u;
  const unsigned want = pass == 0 ? 0u : above_of(state[bh].prefix, pass);
  __syncthreads();
  const float* in = scores + bh * g2;
  for (int c = 0; c < kChunksPerGroup; ++c) {
    const long long base = ((long long)blockIdx.x * kChunksPerGroup + c) * kChunk;
    if (base >= g2) break;
    float x[kKeysPerThread];
#pragma unroll
    for (int i = 0; i < kKeysPerThread; ++i) {
      const long long e = base + i * kHistThreads + threadIdx.x;
      x[i] = e < g2 ? in[e] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kKeysPerThread; ++i) {
      const long long e = base + i * kHistThreads + threadIdx.x;
      const unsigned key = gkey(x[i]);
      bool mine = e < g2 && above_of(key, pass) == want;
      const unsigned dg = digit_of(key, pass);
      // When every lane of the wave holds the same digit (a constant map, say) one lane adds for all: the
      // same-address adds of 64 lanes would go one by one.  Otherwise the digits of one map fall into a few
      // dozen bins at most, and the plain adds cost a few turns each.
      const unsigned long long todo = __ballot(mine);
      const unsigned d0 = (unsigned)__builtin_amdgcn_readfirstlane((int)dg);
      if (todo != 0ull && __ballot(mine && dg != d0) == 0ull && (todo & 1ull)) {
        if ((threadIdx.x & 63) == 0) atomicAdd(&lh[d0], (unsigned)__popcll(todo));
        mine = false;
      }
      if (mine) atomicAdd(&lh[dg], 1u);
    }
  }
  __syncthreads();
  unsigned* out = hist + (bh * 3 + pass) * kBins;
  for (int i = threadIdx.x; i < kBins; i += kHistThreads) {
    const unsigned c = lh[i];
    if (c) atomicAdd(&out[i], c);
  }
}

// One workgroup per head: walk the histogram of this pass from the top bin down to the bin that holds the
// key of the rank looked for; fix the digit, and keep the rank inside that bin.
__global__ __launch_bounds__(256) void resolve_kernel(const unsigned* __restrict__ hist, SelState* __restrict__ state,
                                                      int pass, unsigned budget) {
  __shared__ unsigned part[256];
  const long long bh = blockIdx.x;
  const unsigned* h = hist + (bh * 3 + pass) * kBins;
  const int t = threadIdx.x;
  // thread t takes bins 2047 - 8t down to 2040 - 8t
  unsigned c[8], sum = 0u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    c[i] = h[kBins - 1 - (8 * t + i)];
    sum += c[i];
  }
  part[t] = sum;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {                 // inclusive scan over the threads
    const unsigned add = t >= o ? part[t - o] : 0u;
    __syncthreads();
    part[t] += add;
    __syncthreads();
  }
  const unsigned rank = pass == 0 ? budget : state[bh].rank;   // 1-based, counted from the largest key
  const unsigned prefix = pass == 0 ? 0u : state[bh].prefix;
  const unsigned incl = part[t], before = incl - sum;
  __syncthreads();                                     // everyone has read the state before it changes
  if (before < rank && rank <= incl) {                 // exactly one thread: the counts add up to >= rank
    unsigned acc = before;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (acc < rank && rank <= acc + c[i]) {
        const unsigned bin = (unsigned)(kBins - 1 - (8 * t + i));
        SelState s;
        s.prefix = prefix | (pass == 0 ? bin << 21 : pass == 1 ? bin << 10 : bin);
        s.rank = rank - acc;
        state[bh] = s;
      }
      acc += c[i];
    }
  }
}

// One wavefront per row: how many keys of the row are above the threshold key, how many equal it.
__global__ __launch_bounds__(64) void count_rows_kernel(const float* __restrict__ scores, const SelState* __restrict__ state,
                                                        int32_t* __restrict__ above, int32_t* __restrict__ equal, int g) {
  const long long row = blockIdx.x;
  const long long bh = row / g;
  const int lane = threadIdx.x;
  const unsigned thr = state[bh].prefix;
  const float* in = scores + row * g;
  int gt = 0, eq = 0;
  for (int j0 = 0; j0 < g; j0 += 256) {
    float x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + 64 * i + lane;
      x[i] = j < g ? in[j] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + 64 * i + lane;
      const unsigned key = gkey(x[i]);
      gt += __popcll(__ballot(j < g && key > thr));
      eq += __popcll(__ballot(j < g && key == thr));
    }
  }
  if (lane == 0) {
    above[row] = gt;
    equal[row] = eq;
  }
}

// One workgroup per head.  need = budget - (keys above the threshold) keys equal to it are taken, in
// row-major order; a row with nothing keeps one column.  row_ptr[bh][0..g] = offsets of the rows' lists.
__global__ __launch_bounds__(256) void scan_rows_kernel(const int32_t* __restrict__ above, const int32_t* __restrict__ equal,
                                                        int32_t* __restrict__ row_ptr, int g, unsigned budget, int cap) {
  __shared__ int buf_a[256], buf_b[256];
  __shared__ int carry[2];
  const long long bh = blockIdx.x;
  const int t = threadIdx.x;
  const int32_t* gt = above + bh * g;
  const int32_t* eq = equal + bh * g;
  int32_t* out = row_ptr + bh * (g + 1);
  // total above the threshold
  int s = 0;
  for (int i = t; i < g; i += 256) s += gt[i];
  buf_a[t] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (t < o) buf_a[t] += buf_a[t + o];
    __syncthreads();
  }
  const int need = (int)budget - buf_a[0];             // > 0: fewer than `budget` keys are above the key of that rank
  __syncthreads();
  if (t == 0) {
    carry[0] = 0;                                      // keys equal to the threshold in the rows before
    carry[1] = 0;                                      // entries in the rows before
    out[0] = 0;
  }
  __syncthreads();
  for (int r0 = 0; r0 < g; r0 += 256) {
    const int r = r0 + t;
    const int my_eq = r < g ? eq[r] : 0;
    const int my_gt = r < g ? gt[r] : 0;
    // inclusive scan of the equal counts
    buf_a[t] = my_eq;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
      const int add = t >= o ? buf_a[t - o] : 0;
      __syncthreads();
      buf_a[t] += add;
      __syncthreads();
    }
    const int eq_before = carry[0] + buf_a[t] - my_eq;
    int take = need - eq_before;
    take = take < 0 ? 0 : take > my_eq ? my_eq : take;
    int cnt = my_gt + take;
    if (r < g && cnt == 0) cnt = 1;                    // the row keeps its best column
    if (r >= g) cnt = 0;
    buf_b[t] = cnt;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
      const int add = t >= o ? buf_b[t - o] : 0;
      __syncthreads();
      buf_b[t] += add;
      __syncthreads();
    }
    if (r < g) out[r + 1] = min(carry[1] + buf_b[t], cap);   // (budget + g <= cap: the bound never binds on counts that add up)
    __syncthreads();
    if (t == 255) {
      carry[0] += buf_a[255];
      carry[1] += buf_b[255];
    }
    __syncthreads();
  }
}

// One wavefront per row: write the kept columns in ascending order at the row's offset.  KPL > 0: the row
// (at most 64 KPL columns) is read once and its keys stay in registers, lane l holding columns l, l + 64, ...;
// KPL == 0: rows of any length, read again where needed.
// The counts of the row (above / equal to the threshold) say what it keeps: everything from the threshold
// up, everything above it, or (the one row per head where the budget runs out among equal keys, or a row
// that keeps only its best column) the keys above plus the first few equal ones.
template <int KPL>
__global__ __launch_bounds__(64) void fill_rows_kernel(const float* __restrict__ scores, const SelState* __restrict__ state,
                                                       const int32_t* __restrict__ above, const int32_t* __restrict__ equal,
                                                       const int32_t* __restrict__ row_ptr, int32_t* __restrict__ cols,
                                                       uint8_t* __restrict__ mask, int g, long long cap) {
  const long long row = blockIdx.x;
  const long long bh = row / g;
  const int i_row = (int)(row - bh * g);
  const int lane = threadIdx.x;
  const float* in = scores + row * g;
  unsigned key[KPL > 0 ? KPL : 1];
  if (KPL > 0) {
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
      const int j = lane + 64 * i;
      key[i] = j < g ? gkey(in[j]) : 0u;              // a column past the end: key 0
    }
  }
  auto key_at = [&](int i) -> unsigned {              // key of column lane + 64 i (0 past the end)
    if (KPL > 0) return key[i];
    const int j = lane + 64 * i;
    return j < g ? gkey(in[j]) : 0u;
  };
  const int n_it = (g + 63) >> 6;
  const int32_t* rp = row_ptr + bh * (g + 1) + i_row;
  const int begin = rp[0], cnt = rp[1] - rp[0];
  int32_t* out = cols + bh * cap + begin;
  uint8_t* mrow = mask ? mask + row * g : nullptr;
  unsigned thr = state[bh].prefix;
  const int gt = above[row], eq = equal[row];
  int need_eq = cnt - gt;                              // keys equal to the threshold that this row takes (its first ones)
  bool in_order = need_eq != 0 && need_eq != eq;       // some of the equal keys, but not all: go by column order
  if (gt + eq == 0) {                                  // nothing reaches the threshold: the first of the row's best
    unsigned best = 0u;
    if (KPL > 0) {
#pragma unroll
      for (int i = 0; i < KPL; ++i) best = max(best, key[i]);
    } else {
      for (int i = 0; i < n_it; ++i) best = max(best, key_at(i));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = max(best, (unsigned)__shfl_xor((int)best, o));
    thr = best;
    need_eq = 1;
    in_order = true;
  }
  // all equal keys, or none of them: one comparison per key.  (A threshold key of 0 is a NaN's: then the
  // columns past the end, whose key is 0 too, need the careful path.)
  const unsigned lo = need_eq == 0 ? thr + 1u : thr;
  if (lo == 0u) in_order = true;
  int written = 0, eq_seen = 0;
  auto place_fast = [&](int i) {
    const int j = lane + 64 * i;
    const bool take = key_at(i) >= lo;
    const unsigned long long take_mask = __ballot(take);
    const int at = written + lanes_below(take_mask);
    if (take && at < cnt) out[at] = j;                 // (at < cnt always holds: the offsets were made from the same counts)
    if (mrow && j < g) mrow[j] = take ? 1 : 0;
    written += __popcll(take_mask);
  };
  auto place_in_order = [&](int i) {
    const int j = lane + 64 * i;
    const unsigned kk = key_at(i);
    const bool is_gt = j < g && kk > thr;
    const bool is_eq = j < g && kk == thr;
    const unsigned long long eq_mask = __ballot(is_eq);
    const bool take = is_gt || (is_eq && eq_seen + lanes_below(eq_mask) < need_eq);
    const unsigned long long take_mask = __ballot(take);
    const int at = written + lanes_below(take_mask);
    if (take && at < cnt) out[at] = j;
    if (mrow && j < g) mrow[j] = take ? 1 : 0;
    written += __popcll(take_mask);
    eq_seen += __popcll(eq_mask);
  };
  if (!in_order) {
    if (KPL > 0) {
#pragma unroll
      for (int i = 0; i < KPL; ++i) {
        if (i >= n_it) break;                          // uniform
        place_fast(i);
      }
    } else {
      for (int i = 0; i < n_it; ++i) place_fast(i);
    }
  } else {
    if (KPL > 0) {
#pragma unroll
      for (int i = 0; i < KPL; ++i) {
        if (i >= n_it) break;
        place_in_order(i);
      }
    } else {
      for (int i = 0; i < n_it; ++i) place_in_order(i);
    }
  }
}

}  // namespace

size_t select_global_workspace(const Geo& q) {
  const size_t bh = (size_t)q.B * q.H;
  return 256 + bh * 3 * kBins * sizeof(unsigned) + ((bh * sizeof(SelState) + 255) & ~(size_t)255) +
         2 * ((bh * (size_t)q.g * sizeof(int32_t) + 255) & ~(size_t)255);
}

hipError_t launch_select_global(const Geo& q, long long budget, long long cap, const float* scores, int32_t* row_ptr,
                                int32_t* cols, uint8_t* mask, void* ws, hipStream_t s) {
  const long long bh = (long long)q.B * q.H;
  const long long g2 = (long long)q.g * q.g;
  char* base = (char*)ws;
  unsigned* hist = (unsigned*)base;
  size_t off = (size_t)bh * 3 * kBins * sizeof(unsigned);
  SelState* state = (SelState*)(base + off);
  off += ((size_t)bh * sizeof(SelState) + 255) & ~(size_t)255;
  int32_t* above = (int32_t*)(base + off);
  off += ((size_t)bh * q.g * sizeof(int32_t) + 255) & ~(size_t)255;
  int32_t* equal = (int32_t*)(base + off);
  const long long words = bh * 3 * kBins + bh * 2;     // the histograms and, right behind them, the search state
  hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s, hist, words);
  const long long per_group = (long long)kChunk * kChunksPerGroup;
  const unsigned chunks = (unsigned)((g2 + per_group - 1) / per_group);
  for (int pass = 0; pass < 3; ++pass) {
    const dim3 grid(chunks, (unsigned)bh);
    if (pass == 0) hipLaunchKernelGGL(hist_kernel<0>, grid, dim3(kHistThreads), 0, s, scores, hist, state, g2);
    if (pass == 1) hipLaunchKernelGGL(hist_kernel<1>, grid, dim3(kHistThreads), 0, s, scores, hist, state, g2);
    if (pass == 2) hipLaunchKernelGGL(hist_kernel<2>, grid, dim3(kHistThreads), 0, s, scores, hist, state, g2);
    hipLaunchKernelGGL(resolve_kernel, dim3((unsigned)bh), dim3(256), 0, s, hist, state, pass, (unsigned)budget);
  }
  const unsigned rows = (unsigned)(bh * q.g);
  hipLaunchKernelGGL(count_rows_kernel, dim3(rows), dim3(64), 0, s, scores, state, above, equal, q.g);
  hipLaunchKernelGGL(scan_rows_kernel, dim3((unsigned)bh), dim3(256), 0, s, above, equal, row_ptr, q.g, (unsigned)budget,
                     (int)cap);
  auto fill = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(rows), dim3(64), 0, s, scores, state, above, equal, row_ptr, cols, mask, q.g, cap);
  };
  if (q.g <= 64 * 16) fill(fill_rows_kernel<16>);
  else if (q.g <= 64 * 32) fill(fill_rows_kernel<32>);
  else if (q.g <= 64 * 64) fill(fill_rows_kernel<64>);
  else fill(fill_rows_kernel<0>);
  return hipGetLastError();
}

}  // namespace da
