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
#include <mutex>
#include "da_internal.h"

// Scratch of the entry point that allocates nothing (da_select_blocks_global_static): one copy per device, held from
// the moment the library's code is loaded on a device until the process ends.  Host code never uses this name as an
// address: static_scratch() asks the runtime for the device address, once per device.
static __device__ __align__(256) unsigned char scratch[DA_STATIC_SCRATCH_BYTES];

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

// One wavefront per row: how many keys of the row are above the threshold key, how many equal it, and which:
// bit l of word i of the row's two bit masks is column 64 i + l.  For a row that nothing of reaches the
// threshold, the column of its best key (the lowest one on ties) as well.
__global__ __launch_bounds__(64) void count_rows_kernel(const float* __restrict__ scores, const SelState* __restrict__ state,
                                                        int32_t* __restrict__ above, int32_t* __restrict__ equal,
                                                        unsigned long long* __restrict__ gt_bits,
                                                        unsigned long long* __restrict__ eq_bits, int32_t* __restrict__ forced,
                                                        int g, int W) {
  const long long row = blockIdx.x;
  const long long bh = row / g;
  const int lane = threadIdx.x;
  const unsigned thr = state[bh].prefix;
  const float* in = scores + row * g;
  int gt = 0, eq = 0;
  unsigned best = 0u;
  unsigned long long my_gt = 0ull, my_eq = 0ull;       // lane l keeps word 64 k + l of the current group of 64 words
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
      const int wi = (j0 >> 6) + i;                     // word of this step (the same in every lane)
      const unsigned key = j < g ? gkey(x[i]) : 0u;
      const unsigned long long bgt = __ballot(j < g && key > thr);
      const unsigned long long beq = __ballot(j < g && key == thr);
      gt += __popcll(bgt);
      eq += __popcll(beq);
      best = max(best, key);
      if ((wi & 63) == lane) {
        my_gt = bgt;
        my_eq = beq;
      }
      if (wi < W && ((wi & 63) == 63 || wi == W - 1)) {  // a group of words is complete: one coalesced store
        const int mine = (wi & ~63) + lane;
        if (mine <= wi) {
          gt_bits[row * W + mine] = my_gt;
          eq_bits[row * W + mine] = my_eq;
        }
      }
    }
  }
  if (lane == 0) {
    above[row] = gt;
    equal[row] = eq;
  }
  if (gt + eq == 0) {                                   // (the same in every lane)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) best = max(best, (unsigned)__shfl_xor((int)best, o));
    for (int j0 = 0; j0 < g; j0 += 64) {
      const int j = j0 + lane;
      const unsigned long long hit = __ballot(j < g && gkey(in[j]) == best);
      if (hit) {
        if (lane == 0) forced[row] = j0 + (int)__builtin_ctzll(hit);
        break;
      }
    }
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

// exclusive prefix sum over the 64 lanes; *total receives the sum
__device__ inline int lane_scan(int v, int lane, int* total) {
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(inc, o);
    if (lane >= o) inc += up;
  }
  *total = __shfl(inc, 63);
  return inc - v;
}

// One wavefront per row: write the kept columns in ascending order at the row's offset, from the row's bit
// masks (the scores are not read again).  Lane l takes word l of a group of 64 words: the keys above the
// threshold, and of the equal ones the row's first need_eq, counted across the words by a lane scan.
__global__ __launch_bounds__(64) void fill_rows_kernel(const int32_t* __restrict__ above, const int32_t* __restrict__ equal,
                                                       const unsigned long long* __restrict__ gt_bits,
                                                       const unsigned long long* __restrict__ eq_bits,
                                                       const int32_t* __restrict__ forced, const int32_t* __restrict__ row_ptr,
                                                       int32_t* __restrict__ cols, uint8_t* __restrict__ mask, int g, int W,
                                                       long long cap) {
  const long long row = blockIdx.x;
  const long long bh = row / g;
  const int i_row = (int)(row - bh * g);
  const int lane = threadIdx.x;
  const int32_t* rp = row_ptr + bh * (g + 1) + i_row;
  const int begin = rp[0], cnt = rp[1] - rp[0];
  int32_t* out = cols + bh * cap + begin;
  uint8_t* mrow = mask ? mask + row * g : nullptr;
  const int gt = above[row], eq = equal[row];
  const int need_eq = cnt - gt;
  const bool only_best = gt + eq == 0;                  // nothing reaches the threshold: the row keeps its best column
  const int best_col = only_best ? forced[row] : -1;
  if (only_best && lane == 0 && cnt > 0) out[0] = best_col;
  int written = 0, eq_seen = 0;
  for (int w0 = 0; w0 < W; w0 += 64) {
    const int wi = w0 + lane;
    unsigned long long G = 0ull, E = 0ull;
    if (wi < W && !only_best) {
      G = gt_bits[row * W + wi];
      E = eq_bits[row * W + wi];
    }
    const int pe = __popcll(E);
    int pe_total;
    const int eq_before = eq_seen + lane_scan(pe, lane, &pe_total);
    int n = need_eq - eq_before;
    n = n < 0 ? 0 : n > pe ? pe : n;
    unsigned long long Et = E;
    if (n < pe) {                                       // the word where the row's share of the equal keys runs out
      Et = 0ull;
      unsigned long long rest = E;
      for (int t = 0; t < n; ++t) {
        Et |= rest & (0ull - rest);
        rest &= rest - 1ull;
      }
    }
    unsigned long long T = G | Et;
    if (only_best && wi == (best_col >> 6)) T = 1ull << (best_col & 63);
    const int pt = only_best ? 0 : __popcll(T);
    int pt_total;
    int at = written + lane_scan(pt, lane, &pt_total);
    if (!only_best) {
      unsigned long long rest = T;
      while (rest) {
        const int bit = (int)__builtin_ctzll(rest);
        rest &= rest - 1ull;
        if (at < cnt) out[at] = 64 * wi + bit;          // (at < cnt always holds: the offsets were made from the same counts)
        ++at;
      }
    }
    if (mrow && wi < W)
      for (int bit = 0; bit < 64 && 64 * wi + bit < g; ++bit) mrow[64 * wi + bit] = (uint8_t)((T >> bit) & 1ull);
    written += pt_total;
    eq_seen += pe_total;
  }
}

}  // namespace

namespace {
inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
}  // namespace

// histograms + search state, the rows' counts, their two bit masks, the best column of rows under the threshold
size_t select_global_workspace(const Geo& q) {
  const size_t bh = (size_t)q.B * q.H, rows = bh * (size_t)q.g, W = ((size_t)q.g + 63) / 64;
  return 256 + up256(bh * 3 * kBins * sizeof(unsigned) + bh * sizeof(SelState)) + 3 * up256(rows * sizeof(int32_t)) +
         2 * up256(rows * W * sizeof(unsigned long long));
}

// Device address of `scratch` on the current device (looked up on the first call on each device).
hipError_t static_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex lock;
  static void* known[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(lock);
  if (!known[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    known[dev] = p;
  }
  *ptr = known[dev];
  return hipSuccess;
}

hipError_t launch_select_global(const Geo& q, long long budget, long long cap, const float* scores, int32_t* row_ptr,
                                int32_t* cols, uint8_t* mask, void* ws, hipStream_t s) {
  const long long bh = (long long)q.B * q.H;
  const long long g2 = (long long)q.g * q.g;
  const size_t rows_n = (size_t)bh * q.g;
  const int W = (q.g + 63) / 64;
  char* base = (char*)ws;
  unsigned* hist = (unsigned*)base;
  SelState* state = (SelState*)(base + (size_t)bh * 3 * kBins * sizeof(unsigned));   // right behind the histograms
  size_t off = up256((size_t)bh * 3 * kBins * sizeof(unsigned) + (size_t)bh * sizeof(SelState));
  int32_t* above = (int32_t*)(base + off);
  off += up256(rows_n * sizeof(int32_t));
  int32_t* equal = (int32_t*)(base + off);
  off += up256(rows_n * sizeof(int32_t));
  int32_t* forced = (int32_t*)(base + off);
  off += up256(rows_n * sizeof(int32_t));
  unsigned long long* gt_bits = (unsigned long long*)(base + off);
  off += up256(rows_n * W * sizeof(unsigned long long));
  unsigned long long* eq_bits = (unsigned long long*)(base + off);
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
  const unsigned rows = (unsigned)rows_n;
  hipLaunchKernelGGL(count_rows_kernel, dim3(rows), dim3(64), 0, s, scores, state, above, equal, gt_bits, eq_bits, forced, q.g,
                     W);
  hipLaunchKernelGGL(scan_rows_kernel, dim3((unsigned)bh), dim3(256), 0, s, above, equal, row_ptr, q.g, (unsigned)budget,
                     (int)cap);
  hipLaunchKernelGGL(fill_rows_kernel, dim3(rows), dim3(64), 0, s, above, equal, gt_bits, eq_bits, forced, row_ptr, cols, mask,
                     q.g, W, cap);
  return hipGetLastError();
}

}  // namespace da
