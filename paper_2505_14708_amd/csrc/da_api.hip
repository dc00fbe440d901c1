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
  if (p->keep_blocks == 0 && !(p->sparsity >= 0.0 && p->sparsity < 1.0)) return DA_ERR_DIM;  // also rejects NaN
  if ((long long)p->ph * p->pw > 4096) return DA_ERR_DIM;
  Geo q;
  q.B = p->B; q.H = p->H; q.T = p->T; q.fh = p->fh; q.fw = p->fw; q.d = p->d;
  q.ph = p->ph; q.pw = p->pw; q.dtype = p->dtype;
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
  *out = q;
  return DA_OK;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

inline size_t elem_size(const Geo& q) { return q.dtype == DA_BF16 ? 2 : 4; }

// row bytes must be a whole number of 16-byte chunks for the vector moves
inline bool row_ok(const Geo& q) { return ((size_t)q.d * elem_size(q)) % 16 == 0; }

inline bool attn_supported(const Geo& q) {
  if (q.dtype == DA_BF16) return (q.block == 64 || q.block == 128) && q.d == 128 && attn_bf16_ring_fits(q) != 0;
  return q.block == 64 && (q.d == 64 || q.d == 128);
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
  size_t qp, kp, vt, op, q_pool, k_pool, logits, idx, total;
};

Workspace plan_workspace(const Geo& q) {
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
  w.logits = off; off += align_up(bh * (size_t)q.g * q.g * sizeof(float));
  w.idx = off; off += align_up(bh * (size_t)q.g * q.k * sizeof(int32_t));
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
  return hip_status(launch_select(q, scores, idx, mask, (hipStream_t)stream));
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
  if (q.dtype == DA_BF16) return hip_status(launch_attn_bf16_ring(q, Qp, Kp, Vt, idx, Op, lse, false, s));
  return hip_status(launch_attn_f32(q, (const float*)Qp, (const float*)Kp, (const float*)Vt, idx, (float*)Op, lse, s));
}

int da_forward(const da_problem* p, const void* Q, const void* K, const void* V, void* O, int32_t* idx_out,
               void* ws, size_t ws_bytes, void* stream) {
  Geo q;
  int st = check_problem(p, &q);
  if (st != DA_OK) return st;
  if (!Q || !K || !V || !O || !ws) return DA_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(idx_out) ||
      ((uintptr_t)ws & 255u) != 0)
    return DA_ERR_ALIGN;
  if (!attn_supported(q) || !row_ok(q)) return DA_ERR_UNSUPPORTED;
  Workspace w = plan_workspace(q);
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
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  // Definition 3.2: pooled Q~, K~ and the draft logits (the ranking of a row of the draft
  // map is the ranking of its logits, so the softmax itself is not needed here)
  if (q.dtype == DA_BF16) {
    // The pooling pass also writes the reordered K of Algorithm 1 (one read of K for both).  Q is
    // not copied at all: the attention kernel reads its query rows from their original places and
    // writes O's rows back to theirs, which is Algorithm 1 for Q and Algorithm 2 for O done by
    // addressing (a row of 256 bytes is contiguous in either order).
    if ((e = launch_pool_reorder(q, Q, K, q_pool, k_pool, nullptr, kp, s)) != hipSuccess) return DA_ERR_HIP;
    if ((e = launch_draft_logits(q, q_pool, k_pool, logits, s)) != hipSuccess) return DA_ERR_HIP;
    if ((e = launch_select(q, logits, idx, nullptr, s)) != hipSuccess) return DA_ERR_HIP;
    if ((e = launch_permute(q, V, vt, DA_REORDER_VOP, s)) != hipSuccess) return DA_ERR_HIP;
    return hip_status(launch_attn_bf16_ring(q, Q, kp, vt, idx, O, nullptr, true, s));
  }
  if ((e = launch_pool_reorder(q, Q, K, q_pool, k_pool, qp, kp, s)) != hipSuccess) return DA_ERR_HIP;
  if ((e = launch_draft_logits(q, q_pool, k_pool, logits, s)) != hipSuccess) return DA_ERR_HIP;
  if ((e = launch_select(q, logits, idx, nullptr, s)) != hipSuccess) return DA_ERR_HIP;
  // Algorithm 1: reorder V (block-transposed)
  if ((e = launch_permute(q, V, vt, DA_REORDER_VT, s)) != hipSuccess) return DA_ERR_HIP;
  // SparseAttn
  e = launch_attn_f32(q, (const float*)qp, (const float*)kp, (const float*)vt, idx, (float*)op, nullptr, s);
  if (e != hipSuccess) return DA_ERR_HIP;
  // Algorithm 2: restore
  return hip_status(launch_permute(q, op, O, DA_RESTORE, s));
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
    default: return "unknown status";
  }
}

}  // extern "C"
