// Host side of the C ABI: argument checks, derived sizes, dispatch to the kernel launchers.
#include <math.h>
#include "da_internal.h"

using namespace da;

namespace {

const long long kMaxInt = 2147483647LL;

int check_problem(const da_problem* p, Geo* out) {
  if (!p) return DA_ERR_NULL;
  if (p->B < 1 || p->H < 1 || p->T < 1 || p->fh < 1 || p->fw < 1 || p->d < 1 || p->ph < 1 || p->pw < 1)
    return DA_ERR_DIM;
  if (p->dtype != DA_F32 && p->dtype != DA_BF16) return DA_ERR_DIM;
  if (p->keep_blocks < 0) return DA_ERR_DIM;
  if (p->pool != DA_POOL_AVG && p->pool != DA_POOL_MAX) return DA_ERR_DIM;
  if (p->keep_blocks == 0 && !(p->sparsity >= 0.0 && p->sparsity < 1.0)) return DA_ERR_DIM;  // also rejects NaN
  if ((long long)p->ph * p->pw > 4096) return DA_ERR_DIM;
  Geo q;
  q.B = p->B; q.H = p->H; q.T = p->T; q.fh = p->fh; q.fw = p->fw; q.d = p->d;
  q.ph = p->ph; q.pw = p->pw; q.dtype = p->dtype; q.pool = p->pool;
  q.gh = (p->fh + p->ph - 1) / p->ph;
  q.gw = (p->fw + p->pw - 1) / p->pw;
  long long g = (long long)p->T * q.gh * q.gw;
  long long block = (long long)p->ph * p->pw;
  long long n = (long long)p->T * p->fh * p->fw;
  long long n_pad = g * block;
  long long bh = (long long)p->B * p->H;
  if (g > (1 << 22) || n_pad > kMaxInt || n > kMaxInt || bh > kMaxInt || bh * g > kMaxInt) return DA_ERR_DIM;
  if ((double)bh * (double)n_pad * (double)p->d > 4.0e15) return DA_ERR_DIM;
  if ((double)bh * (double)g * (double)g > 4.0e15) return DA_ERR_DIM;
  q.g = (int)g; q.block = (int)block; q.n = n; q.n_pad = n_pad;
  long long k;
  if (p->keep_blocks > 0) {
    k = p->keep_blocks;
  } else {
    // the paper's r is the kept fraction; `sparsity` is the dropped one (Table 1's Sparse Ratio)
    k = g - (long long)floor(p->sparsity * (double)g + 1e-6);
  }
  if (k < 1) k = 1;
  if (k > g) k = g;
  q.k = (int)k;
  // contiguous [B, H, N, d] in the original order unless an entry point says otherwise
  q.in.sn = q.d; q.in.sh = q.n * q.d; q.in.sb = (long long)q.H * q.n * q.d;
  q.out = q.in;
  q.reordered = 0;
  *out = q;
  return DA_OK;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

inline size_t elem_size(const Geo& q) { return q.dtype == DA_BF16 ? 2 : 4; }

// row bytes must be a whole number of 16-byte chunks for the vector moves
inline bool row_ok(const Geo& q) { return ((size_t)q.d * elem_size(q)) % 16 == 0; }

inline bool attn_supported(const Geo& q, bool any_length = false) {
  if (q.dtype == DA_BF16)
    return (q.block == 64 || q.block == 128) && q.d == 128 && attn_bf16_ring_fits(q, any_length) != 0;
  return q.block == 64 && (q.d == 64 || q.d == 128);
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Entries kept by the whole-map selection (Section 3.2.2: ceil(r g^2), here g^2 - floor(sparsity g^2 + 1e-6);
// k per row given explicitly means the same total, k g) and the room to allocate per (batch, head): a row the
// threshold leaves empty keeps one column, so up to g more.  Returns false when the offsets do not fit int32
// (or a head's map has 2^32 entries or more).
bool global_budget(const da_problem* p, const Geo& q, long long* budget, long long* cap) {
  const long long g2 = (long long)q.g * q.g;
  if (g2 > 0xffffffffLL) return false;                 // the selector counts the keys of a head in 32 bits
  long long b = p->keep_blocks > 0 ? (long long)q.k * q.g : g2 - (long long)floor(p->sparsity * (double)g2 + 1e-6);
  if (b < 1) b = 1;
  if (b > g2) b = g2;
  *budget = b;
  *cap = (b + q.g + 3) & ~3LL;                         // heads' lists stay 16-byte aligned
  return *cap <= kMaxInt && (double)q.B * q.H * (double)*cap < 4.0e15;
}

struct Workspace {
  size_t qp, kp, vt, op, q_pool, k_pool, logits, idx, row_ptr, select, total;
};

// lists_cap > 0: the whole-map selection (lists of any length, `lists_cap` entries per head) instead of k per row
Workspace plan_workspace(const Geo& q, long long lists_cap = 0) {
  Workspace w;
  size_t bh = (size_t)q.B * q.H;
  size_t big = align_up(bh * (size_t)q.n_pad * q.d * elem_size(q));
  size_t pooled = align_up(bh * (size_t)q.g * q.d * sizeof(float));
  // the bf16 attention kernel reads Q and writes O in the original token order: no reordered copies of them
  const bool direct = q.dtype == DA_BF16;
  size_t off = 0;
  w.qp = off; off += direct ? 0 : big;
  w.kp = off; off += big;
  w.vt = off; off += big;
  w.op = off; off += direct ? 0 : big;
  w.q_pool = off; off += pooled;
  w.k_pool = off; off += pooled;
  w.logits = off; off += align_up(bh * (size_t)q.g * q.g * sizeof(float) + kSelectSlack);   // (the selector may read on past a row's end)
  w.idx = off; off += align_up(bh * (lists_cap > 0 ? (size_t)lists_cap : (size_t)q.g * q.k) * sizeof(int32_t));
  w.row_ptr = off; off += lists_cap > 0 ? align_up(bh * ((size_t)q.g + 1) * sizeof(int32_t)) : 0;
  w.select = off; off += lists_cap > 0 ? align_up(select_global_workspace(q)) : 0;
  w.total = off;
  return w;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? DA_OK : DA_ERR_HIP; }

}  // namespace

extern "C" {

int da_derive(const da_problem* p, da_dims* out) {
  if (!out) return DA_ERR_NULL;
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  out->gh = q.gh; out->gw = q.gw; out->g = q.g; out->block = q.block; out->k = q.k;
  out->reserved = 0; out->n = q.n; out->n_pad = q.n_pad;
  return DA_OK;
}

int da_workspace_size(const da_problem* p, size_t* bytes) {
  if (!bytes) return DA_ERR_NULL;
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  *bytes = plan_workspace(q).total;
  return DA_OK;
}

int da_build_perm(const da_problem* p, int32_t* perm, int32_t* inv, int32_t* valid, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (misaligned(perm) || misaligned(inv) || misaligned(valid)) return DA_ERR_ALIGN;
  return hip_status(launch_build_perm(q, perm, inv, valid, (hipStream_t)stream));
}

int da_draft_map(const da_problem* p, const void* Q, const void* K, float* q_pool, float* k_pool,
                 float* logits, float* draft, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!Q || !K || !q_pool || !k_pool) return DA_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(q_pool) || misaligned(k_pool) || misaligned(logits) ||
      misaligned(draft))
    return DA_ERR_ALIGN;
  if (!row_ok(q)) return DA_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = launch_pool(q, Q, K, q_pool, k_pool, s);
  if (e != hipSuccess) return DA_ERR_HIP;
  if (logits || draft) {
    // the map needs the logits; when the caller does not want them they live in `draft`
    float* L = logits ? logits : draft;
    e = launch_draft_logits(q, q_pool, k_pool, L, s);
    if (e != hipSuccess) return DA_ERR_HIP;
    if (draft) e = launch_row_softmax(q, L, draft, s);
  }
  return hip_status(e);
}

int da_select_blocks(const da_problem* p, const float* scores, int32_t* idx, uint8_t* mask, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!scores || !idx) return DA_ERR_NULL;
  if (misaligned(scores) || misaligned(idx) || misaligned(mask)) return DA_ERR_ALIGN;
  return hip_status(launch_select(q, scores, idx, mask, false, (hipStream_t)stream));
}

int da_permute(const da_problem* p, const void* X, void* Y, int mode, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!X || !Y) return DA_ERR_NULL;
  if (mode != DA_REORDER_ROWS && mode != DA_REORDER_VT && mode != DA_RESTORE && mode != DA_REORDER_VOP) return DA_ERR_DIM;
  if (misaligned(X) || misaligned(Y)) return DA_ERR_ALIGN;
  if (!row_ok(q)) return DA_ERR_UNSUPPORTED;
  if (mode == DA_REORDER_VT && ((size_t)q.block * elem_size(q)) % 16 != 0) return DA_ERR_UNSUPPORTED;
  if (mode == DA_REORDER_VOP && (q.dtype != DA_BF16 || q.block % 64 != 0 || q.d % 32 != 0)) return DA_ERR_UNSUPPORTED;
  return hip_status(launch_permute(q, X, Y, mode, (hipStream_t)stream));
}

int da_sparse_attn(const da_problem* p, const void* Qp, const void* Kp, const void* Vt, const int32_t* idx,
                   void* Op, float* lse, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!Qp || !Kp || !Vt || !idx || !Op) return DA_ERR_NULL;
  if (misaligned(Qp) || misaligned(Kp) || misaligned(Vt) || misaligned(idx) || misaligned(Op) || misaligned(lse))
    return DA_ERR_ALIGN;
  if (!attn_supported(q)) return DA_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (q.dtype == DA_BF16)
    return hip_status(launch_attn_bf16_ring(q, Qp, Kp, Vt, idx, nullptr, 0, Op, lse, false, nullptr, s));
  return hip_status(
      launch_attn_f32(q, (const float*)Qp, (const float*)Kp, (const float*)Vt, idx, nullptr, 0, (float*)Op, lse, s));
}

int da_sparse_attn_ex(const da_problem* p, const void* Q, const void* Kp, const void* Vt, const int32_t* idx, void* O,
                      float* lse, int original_order, uint64_t* tile_counts, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!Q || !Kp || !Vt || !idx || !O) return DA_ERR_NULL;
  if (original_order != 0 && original_order != 1) return DA_ERR_DIM;
  if (misaligned(Q) || misaligned(Kp) || misaligned(Vt) || misaligned(idx) || misaligned(O) || misaligned(lse) ||
      ((uintptr_t)tile_counts & 7u) != 0)
    return DA_ERR_ALIGN;
  if (!attn_supported(q)) return DA_ERR_UNSUPPORTED;
  if (q.dtype != DA_BF16) {
    if (original_order || tile_counts) return DA_ERR_UNSUPPORTED;
    return hip_status(launch_attn_f32(q, (const float*)Q, (const float*)Kp, (const float*)Vt, idx, nullptr, 0, (float*)O,
                                      lse, (hipStream_t)stream));
  }
  return hip_status(launch_attn_bf16_ring(q, Q, Kp, Vt, idx, nullptr, 0, O, lse, original_order != 0,
                                          (unsigned long long*)tile_counts, (hipStream_t)stream));
}

int da_wait_failures(uint64_t* count) {
  if (!count) return DA_ERR_NULL;
  unsigned long long c = 0ull;
  if (read_wait_failures(&c) != hipSuccess) return DA_ERR_HIP;
  *count = c;
  return DA_OK;
}

// da_forward and da_forward_global: the same launches but for the selection
// in / out: where the caller's Q, K, V and O live (NULL: contiguous); reordered: their rows are the slots of
// Algorithm 1's order instead of tokens
static int set_layout(Geo& q, const da_layout* in, const da_layout* out, int reordered) {
  if (reordered != 0 && reordered != 1) return DA_ERR_DIM;
  q.reordered = reordered;
  const long long rows = reordered ? q.n_pad : q.n;
  const long long per = q.dtype == DA_BF16 ? 8 : 4;   // elements per 16 bytes
  Rows dflt;
  dflt.sn = q.d; dflt.sh = rows * q.d; dflt.sb = (long long)q.H * rows * q.d;
  q.in = q.out = dflt;
  const da_layout* given[2] = {in, out};
  Rows* into[2] = {&q.in, &q.out};
  for (int t = 0; t < 2; ++t) {
    if (!given[t]) continue;
    const da_layout& l = *given[t];
    if (l.stride_n < q.d || l.stride_h < 1 || l.stride_b < 1) return DA_ERR_DIM;
    if (l.stride_n % per || l.stride_h % per || l.stride_b % per) return DA_ERR_ALIGN;
    // the last element must be addressable with 63-bit offsets, with room to spare
    if ((double)q.B * (double)l.stride_b + (double)q.H * (double)l.stride_h + (double)rows * (double)l.stride_n > 4.0e15)
      return DA_ERR_DIM;
    into[t]->sb = l.stride_b; into[t]->sh = l.stride_h; into[t]->sn = l.stride_n;
  }
  return DA_OK;
}

static int forward_impl(const da_problem* p, bool whole_map, const da_layout* in, const da_layout* out, int reordered,
                        const void* Q, const void* K, const void* V, void* O, int32_t* idx_out, int32_t* row_ptr_out,
                        void* ws, size_t ws_bytes, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if ((st = set_layout(q, in, out, reordered)) != DA_OK) return st;
  if (!Q || !K || !V || !O || !ws) return DA_ERR_NULL;
  if (whole_map && (idx_out == nullptr) != (row_ptr_out == nullptr)) return DA_ERR_NULL;   // both or neither
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(idx_out) ||
      misaligned(row_ptr_out) || ((uintptr_t)ws & 255u) != 0)
    return DA_ERR_ALIGN;
  if (!attn_supported(q, whole_map) || !row_ok(q)) return DA_ERR_UNSUPPORTED;
  long long budget = 0, cap = 0;
  if (whole_map && !global_budget(p, q, &budget, &cap)) return DA_ERR_DIM;
  Workspace w = plan_workspace(q, cap);
  if (ws_bytes < w.total) return DA_ERR_WORKSPACE;
  char* base = (char*)ws;
  void* qp = base + w.qp;
  void* kp = base + w.kp;
  void* vt = base + w.vt;
  void* op = base + w.op;
  float* q_pool = (float*)(base + w.q_pool);
  float* k_pool = (float*)(base + w.k_pool);
  float* logits = (float*)(base + w.logits);
  int32_t* idx = idx_out ? idx_out : (int32_t*)(base + w.idx);
  int32_t* row_ptr = !whole_map ? nullptr : row_ptr_out ? row_ptr_out : (int32_t*)(base + w.row_ptr);
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  const bool bf16 = q.dtype == DA_BF16;
  // Definition 3.2: pooled Q~, K~ and the draft logits (the ranking of a row of the draft
  // map is the ranking of its logits, so the softmax itself is not needed here).
  // The pooling pass also writes the reordered K of Algorithm 1 (one read of K for both).  With bf16, Q is
  // not copied at all: the attention kernel reads its query rows from their original places and
  // writes O's rows back to theirs, which is Algorithm 1 for Q and Algorithm 2 for O done by
  // addressing (a row of 256 bytes is contiguous in either order).
  // (K that already is a contiguous reordered tensor is used where it is.)
  const bool k_in_place = bf16 && q.reordered && q.in.sn == q.d && q.in.sh == q.n_pad * q.d &&
                          q.in.sb == (long long)q.H * q.n_pad * q.d;
  if (k_in_place) kp = const_cast<void*>(K);
  // Every block kept (sparsity 0, as in the steps Section 4.1 leaves dense): there is nothing to rank.  The lists are
  // 0 .. g-1 whatever the draft map says, so pooling, logits and selection are left out and only Algorithm 1 runs.
  const bool all_kept = whole_map ? budget == (long long)q.g * q.g : q.k == q.g;
  if (all_kept) {
    if (!k_in_place && (e = launch_permute(q, K, kp, DA_REORDER_ROWS, s)) != hipSuccess) return DA_ERR_HIP;
    if (!bf16 && (e = launch_permute(q, Q, qp, DA_REORDER_ROWS, s)) != hipSuccess) return DA_ERR_HIP;
    e = launch_all_lists(q, idx, row_ptr, whole_map ? cap : (long long)q.g * q.g, s);
  } else {
    if ((e = launch_pool_reorder(q, Q, K, q_pool, k_pool, bf16 ? nullptr : qp, k_in_place ? nullptr : kp, s)) !=
        hipSuccess)
      return DA_ERR_HIP;
    if ((e = launch_draft_logits(q, q_pool, k_pool, logits, s)) != hipSuccess) return DA_ERR_HIP;
    // guided sparsity: k per row, or the threshold over the whole map (Section 3.2.2)
    if (whole_map)
      e = launch_select_global(q, budget, cap, logits, row_ptr, idx, nullptr, base + w.select, s);
    else
      e = launch_select(q, logits, idx, nullptr, true, s);
  }
  if (e != hipSuccess) return DA_ERR_HIP;
  // Algorithm 1: reorder V (block-transposed; for bf16 as matrix operands)
  if ((e = launch_permute(q, V, vt, bf16 ? DA_REORDER_VOP : DA_REORDER_VT, s)) != hipSuccess) return DA_ERR_HIP;
  // SparseAttn
  if (bf16) return hip_status(launch_attn_bf16_ring(q, Q, kp, vt, idx, row_ptr, cap, O, nullptr, true, nullptr, s));
  e = launch_attn_f32(q, (const float*)qp, (const float*)kp, (const float*)vt, idx, row_ptr, cap, (float*)op, nullptr, s);
  if (e != hipSuccess) return DA_ERR_HIP;
  // Algorithm 2: restore
  return hip_status(launch_permute(q, op, O, DA_RESTORE, s));
}

int da_forward(const da_problem* p, const void* Q, const void* K, const void* V, void* O, int32_t* idx_out,
               void* ws, size_t ws_bytes, void* stream) {
  return forward_impl(p, false, nullptr, nullptr, 0, Q, K, V, O, idx_out, nullptr, ws, ws_bytes, stream);
}

int da_forward_ex(const da_problem* p, const da_layout* in, const da_layout* out, int reordered, const void* Q,
                  const void* K, const void* V, void* O, int32_t* idx_out, void* ws, size_t ws_bytes, void* stream) {
  return forward_impl(p, false, in, out, reordered, Q, K, V, O, idx_out, nullptr, ws, ws_bytes, stream);
}

int da_global_sizes(const da_problem* p, da_global_dims* out) {
  if (!out) return DA_ERR_NULL;
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  long long budget, cap;
  if (!global_budget(p, q, &budget, &cap)) return DA_ERR_DIM;
  out->budget = budget;
  out->cap = cap;
  out->select_ws = align_up(select_global_workspace(q));
  out->forward_ws = plan_workspace(q, cap).total;
  return DA_OK;
}

int da_select_blocks_global(const da_problem* p, const float* scores, int32_t* row_ptr, int32_t* cols, uint8_t* mask,
                            void* ws, size_t ws_bytes, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!scores || !row_ptr || !cols || !ws) return DA_ERR_NULL;
  if (misaligned(scores) || misaligned(row_ptr) || misaligned(cols) || misaligned(mask) || ((uintptr_t)ws & 255u) != 0)
    return DA_ERR_ALIGN;
  long long budget, cap;
  if (!global_budget(p, q, &budget, &cap)) return DA_ERR_DIM;
  if (ws_bytes < align_up(select_global_workspace(q))) return DA_ERR_WORKSPACE;
  return hip_status(launch_select_global(q, budget, cap, scores, row_ptr, cols, mask, ws, (hipStream_t)stream));
}

int da_select_blocks_global_static(const da_problem* p, const float* scores, int32_t* row_ptr, int32_t* cols,
                                   uint8_t* mask, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!scores || !row_ptr || !cols) return DA_ERR_NULL;
  if (misaligned(scores) || misaligned(row_ptr) || misaligned(cols) || misaligned(mask)) return DA_ERR_ALIGN;
  long long budget, cap;
  if (!global_budget(p, q, &budget, &cap)) return DA_ERR_DIM;
  if (align_up(select_global_workspace(q)) > (size_t)DA_STATIC_SCRATCH_BYTES) return DA_ERR_SCRATCH;
  void* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return DA_ERR_HIP;
  return hip_status(launch_select_global(q, budget, cap, scores, row_ptr, cols, mask, ws, (hipStream_t)stream));
}

int da_sparse_attn_lists(const da_problem* p, const void* Qp, const void* Kp, const void* Vt, const int32_t* row_ptr,
                         const int32_t* cols, int64_t cap, void* Op, float* lse, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!Qp || !Kp || !Vt || !row_ptr || !cols || !Op) return DA_ERR_NULL;
  if (cap < 1 || cap > kMaxInt || (cap & 3) != 0) return DA_ERR_DIM;
  if (misaligned(Qp) || misaligned(Kp) || misaligned(Vt) || misaligned(row_ptr) || misaligned(cols) || misaligned(Op) ||
      misaligned(lse))
    return DA_ERR_ALIGN;
  if (!attn_supported(q, true)) return DA_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (q.dtype == DA_BF16) return hip_status(launch_attn_bf16_ring(q, Qp, Kp, Vt, cols, row_ptr, cap, Op, lse, false, nullptr, s));
  return hip_status(launch_attn_f32(q, (const float*)Qp, (const float*)Kp, (const float*)Vt, cols, row_ptr, cap,
                                    (float*)Op, lse, s));
}

int da_forward_global(const da_problem* p, const void* Q, const void* K, const void* V, void* O, int32_t* row_ptr_out,
                      int32_t* cols_out, void* ws, size_t ws_bytes, void* stream) {
  return forward_impl(p, true, nullptr, nullptr, 0, Q, K, V, O, cols_out, row_ptr_out, ws, ws_bytes, stream);
}

const char* da_status_string(int status) {
  switch (status) {
    case DA_OK: return "ok";
    case DA_ERR_NULL: return "a required pointer is NULL";
    case DA_ERR_DIM: return "bad size, ratio or mode";
    case DA_ERR_UNSUPPORTED: return "no kernel for this window, head dimension or dtype";
    case DA_ERR_WORKSPACE: return "workspace too small";
    case DA_ERR_ALIGN: return "device pointer not aligned";
    case DA_ERR_HIP: return "HIP launch failed";
    case DA_ERR_SCRATCH: return "the problem needs more scratch than the built-in buffer holds";
    default: return "unknown status";
  }
}

}  // extern "C"
