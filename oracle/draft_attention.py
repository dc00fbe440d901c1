"""CPU oracle for the DraftAttention hot path (arxiv 2505.14708).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, NumPy float64 statement of what the
method computes, written from the paper, and it shares no code with the HIP path.  Only
the tests, the smoke check and the bench's ``cpu_baseline`` leg may call it; the product
path never does.

What follows the paper where:

  reorder_index        Algorithm 1 (Generate Reorder Index), plus the padding reading
  restore_index        Algorithm 2 (Generate Restore Index)
  pool_*               Definition 3.2, the two average-pooling equations
  pool_max_f32         the max-pooling kernel of the ablation (Section 4.3): same regions, max instead of mean
  draft_logits_*, draft_map   Definition 3.2, the draft attention map equation
  select_blocks        "Guided Sparsity via Draft Attention" paragraph (top entries kept)
  select_blocks_global the threshold form of the mask, Section 3.2.2 "Error from Sparsity Mask"
                       (t = the ceil(r g^2)-th largest region-level score of the whole map)
  lift_mask            the lifted mask equation  M^_uv = M_ij  (same paragraph)
  permute / restore    Section 3.3, Execution and Restoration paragraphs
  sparse_attention_*   the SparseAttn equation (same paragraph as the mask)
  full_attention       Definition 3.1

Readings taken where the paper is silent or loose (each is listed in the design notes):

  * masked entries are *excluded* from the softmax (probability 0), not multiplied by 0
    inside it: the text says every region is either computed or skipped, and only this
    reading makes 0 % sparsity equal Definition 3.1;
  * ``sparsity`` is the dropped fraction (the "Sparse Ratio" column of Table 1); the
    paper's r is 1 - sparsity;  k = g - floor(sparsity*g + 1e-6), clamped to [1, g];
  * the top entries are taken per query-block row (k per row), ranked on the float32
    draft logits (softmax is monotone per row, so the order is that of A_draft), ties
    to the lowest column index, lists ascending;
  * the whole-map form (select_blocks_global) keeps exactly ceil(r g^2) entries of a head's
    map: with distinct scores that is the paper's {S~_ij >= t}; scores equal to t are taken
    in row-major order until the budget is used up (the per-row tie rule, extended), so the
    size of the result does not depend on the data.  A row that the threshold leaves empty
    keeps its single best column (lowest index on ties): the attention of its queries is
    otherwise undefined.  The budget is g^2 - floor(sparsity*g^2 + 1e-6), or keep_blocks*g
    when keep_blocks is given (the same total as k per row);
  * frames whose size the window does not divide get partial edge patches ("appropriate
    padding", Section 4.1): patches are anchored at (0,0) of each frame, a block holds
    its valid tokens in Algorithm 1's (u, v) raster order first and pad slots (index -1)
    at the tail; pad rows are zeros, pad keys are never attended, pooled means divide by
    the number of valid tokens (the |R_i| of Definition 3.2);
  * the scale is 1/sqrt(d) in both the draft map and the attention.

Float32 "canonical" variants exist because the kept-block decision is an integer taken
from floating point: the HIP path and the oracle both evaluate the draft logits in
float32 with one fixed order of operations (documented at each function), so the
decision can be compared bit for bit.  Everything else is float64, and everything is NumPy
except the chain of fused multiply-adds of the canonical logits, which is the plain C loop in
draft_logits_fma.c (built on first use by build_native()).
"""
from __future__ import annotations

import math
import numpy as np

F32 = 0
BF16 = 1


# ----------------------------------------------------------------------------
# sizes
# ----------------------------------------------------------------------------
def derive_dims(T, fh, fw, ph, pw, sparsity=0.0, keep_blocks=0):
    """Grid of pooled patches and the number k of key blocks kept per query block."""
    gh = -(-fh // ph)
    gw = -(-fw // pw)
    g = T * gh * gw
    block = ph * pw
    if keep_blocks and keep_blocks > 0:
        k = int(keep_blocks)
    else:
        k = g - int(math.floor(sparsity * g + 1e-6))
    k = max(1, min(g, k))
    return dict(gh=gh, gw=gw, g=g, block=block, n=T * fh * fw, n_pad=g * block, k=k)


# ----------------------------------------------------------------------------
# Algorithm 1 / Algorithm 2
# ----------------------------------------------------------------------------
def reorder_index(T, fh, fw, ph, pw):
    """Algorithm 1 with partial edge patches.

    Returns (perm, valid): perm[slot] is the original token stored at ``slot`` of the
    reordered sequence or -1 for a pad slot; valid[i] is the number of real tokens in
    block i.  Loops are those of Algorithm 1 (frame, patch row, patch column, row in
    patch, column in patch); a (u, v) that falls outside the frame is skipped and the
    block is padded at its tail.  When ph | fh and pw | fw nothing is skipped and this
    is Algorithm 1 as printed.
    """
    gh = -(-fh // ph)
    gw = -(-fw // pw)
    block = ph * pw
    perm = []
    valid = []
    for f in range(T):
        for i in range(gh):
            for j in range(gw):
                cnt = 0
                for u in range(ph):
                    for v in range(pw):
                        y = i * ph + u
                        x = j * pw + v
                        if y < fh and x < fw:
                            perm.append(f * fh * fw + y * fw + x)
                            cnt += 1
                perm.extend([-1] * (block - cnt))
                valid.append(cnt)
    return np.asarray(perm, dtype=np.int64), np.asarray(valid, dtype=np.int64)


def restore_index(perm, n):
    """Algorithm 2: inv[perm[i]] = i over the non-pad slots."""
    inv = np.zeros(n, dtype=np.int64)
    for i, p in enumerate(perm):
        if p >= 0:
            inv[p] = i
    return inv


# ----------------------------------------------------------------------------
# storage widening
# ----------------------------------------------------------------------------
def widen_f32(x, dtype):
    """Stored bits -> float32 (exact): float32 as is, bf16 bit patterns shifted up."""
    if dtype == F32:
        return np.asarray(x, dtype=np.float32)
    return (np.asarray(x, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen_f64(x, dtype):
    return widen_f32(x, dtype).astype(np.float64)


# ----------------------------------------------------------------------------
# reorder / restore of a [N, d] tensor
# ----------------------------------------------------------------------------
def permute(X, perm):
    """Xp[slot] = X[perm[slot]], zeros in pad slots.  X is [N, d]; result [n_pad, d]."""
    Xp = np.zeros((len(perm),) + X.shape[1:], dtype=X.dtype)
    ok = perm >= 0
    Xp[ok] = X[perm[ok]]
    return Xp


def restore(Xp, inv):
    """X[n] = Xp[inv[n]]."""
    return Xp[inv]


# ----------------------------------------------------------------------------
# Definition 3.2: pooling
# ----------------------------------------------------------------------------
def pool_f64(X64, perm, valid, block):
    """Mean over the valid tokens of each block, float64.  X64 is [N, d] -> [g, d]."""
    g = len(valid)
    out = np.zeros((g, X64.shape[1]), dtype=np.float64)
    for i in range(g):
        toks = perm[i * block:i * block + valid[i]]
        out[i] = X64[toks].sum(axis=0) / valid[i]
    return out


def pool_canonical_f32(X32, perm, valid, block):
    """The float32 pooling whose bits define the mask.

    Order of operations: acc = 0; for slot = 0 .. valid-1 in block order:
    acc = fl32(acc + x[slot]);  mean = fl32(acc / fl32(valid)).
    """
    g = len(valid)
    d = X32.shape[1]
    acc = np.zeros((g, d), dtype=np.float32)
    pm = perm.reshape(g, block)
    for s in range(block):
        live = valid > s
        if not live.any():
            break
        acc[live] = acc[live] + X32[pm[live, s]]
    return acc / valid.astype(np.float32)[:, None]


def pool_max_f32(X32, perm, valid, block):
    """Max over the valid tokens of each block (the ablation's downsampling kernel, Section 4.3),
    float32 in, float32 out: exact, no rounding.  Taken slot by slot, acc = x if x > acc else acc,
    starting from the block's first token, so a tie between -0 and +0 keeps the earlier one."""
    g = len(valid)
    pm = perm.reshape(g, block)
    acc = X32[pm[:, 0]].astype(np.float32).copy()        # slot 0 of every block is a real token
    for s in range(1, block):
        live = valid > s
        if not live.any():
            break
        x = X32[pm[live, s]]
        acc[live] = np.where(x > acc[live], x, acc[live])
    return acc


# ----------------------------------------------------------------------------
# Definition 3.2: draft map
# ----------------------------------------------------------------------------
def draft_logits_f64(qp64, kp64):
    d = qp64.shape[1]
    return (qp64 @ kp64.T) / math.sqrt(d)


_NATIVE = None


def build_native(force=False):
    """Compile the oracle's one C routine (draft_logits_fma.c, beside this file) into oracle/_build/ and return
    the path of the shared object.  The routine is a plain triple loop around fmaf(); it is in C because an exact
    fused multiply-add cannot be written with NumPy's float32 operations."""
    import os
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    src = os.path.join(here, "draft_logits_fma.c")
    out_dir = os.path.join(here, "_build")
    lib = os.path.join(out_dir, "libdraftoracle.so")
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        os.makedirs(out_dir, exist_ok=True)
        subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-shared", "-fPIC", src, "-o", lib, "-lm"], check=True)
    return lib


def _native():
    global _NATIVE
    if _NATIVE is None:
        import ctypes
        L = ctypes.CDLL(build_native())
        L.da_oracle_draft_logits_fma.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_long] * 3 + [ctypes.c_float]
        L.da_oracle_draft_logits_fma.restype = None
        _NATIVE = L
    return _NATIVE


def draft_logits_canonical_f32(qp32, kp32):
    """Float32 draft logits with a fixed order: acc = 0; for c = 0 .. d-1:
    acc = fma(q[c], k[c], acc) (IEEE fused multiply-add: the exact product plus acc, rounded once);
    L = fl32(acc * fl32(1/sqrt(d))).  Evaluated by the C routine in draft_logits_fma.c."""
    qp32 = np.ascontiguousarray(qp32, dtype=np.float32)
    kp32 = np.ascontiguousarray(kp32, dtype=np.float32)
    g, d = qp32.shape
    out = np.empty((g, kp32.shape[0]), dtype=np.float32)
    scale = np.float32(1.0 / math.sqrt(d))
    _native().da_oracle_draft_logits_fma(qp32.ctypes.data, kp32.ctypes.data, out.ctypes.data, g, kp32.shape[0], d, scale)
    return out


def softmax_rows(L):
    L = np.asarray(L, dtype=np.float64)
    e = np.exp(L - L.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def draft_map(qp64, kp64):
    """A_draft = Softmax(Q~ K~^T / sqrt(d)), float64, [g, g]."""
    return softmax_rows(draft_logits_f64(qp64, kp64))


# ----------------------------------------------------------------------------
# guided sparsity: top-k per row
# ----------------------------------------------------------------------------
def select_blocks(scores, k):
    """Per row keep the k largest scores, ties to the lowest column; ascending lists.

    Returns (idx [g, k] int64 ascending, mask [g, g] uint8).
    """
    scores = np.asarray(scores)
    g_rows, g_cols = scores.shape
    idx = np.empty((g_rows, k), dtype=np.int64)
    mask = np.zeros((g_rows, g_cols), dtype=np.uint8)
    for i in range(g_rows):
        # stable sort of the negated row: descending score, equal scores by column
        order = np.argsort(-scores[i], kind="stable")[:k]
        idx[i] = np.sort(order)
        mask[i, idx[i]] = 1
    return idx, mask


def global_budget(g, sparsity=0.0, keep_blocks=0):
    """Entries of one head's g x g map kept by the whole-map selection: ceil(r g^2)."""
    if keep_blocks and keep_blocks > 0:
        total = int(keep_blocks) * g
    else:
        total = g * g - int(math.floor(sparsity * g * g + 1e-6))
    return max(1, min(g * g, total))


def select_blocks_global(scores, total):
    """Whole-map threshold selection (Section 3.2.2): the ``total`` largest entries of the
    map, equal scores in row-major order; rows left empty keep their best column.

    Returns (row_ptr [g+1] int64, cols int64 (row by row, ascending inside a row),
    mask [g, g] uint8).
    """
    scores = np.asarray(scores)
    g_rows, g_cols = scores.shape
    flat = scores.reshape(-1)
    # stable sort of the negated map: descending score, equal scores by (row, column)
    order = np.argsort(-flat, kind="stable")[:total]
    mask = np.zeros(g_rows * g_cols, dtype=np.uint8)
    mask[order] = 1
    mask = mask.reshape(g_rows, g_cols)
    for i in range(g_rows):
        if not mask[i].any():
            mask[i, int(np.argmax(scores[i]))] = 1          # argmax returns the first of equal maxima
    counts = mask.sum(axis=1, dtype=np.int64)
    row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    cols = np.nonzero(mask)[1].astype(np.int64)             # row-major: row by row, ascending columns
    return row_ptr, cols, mask


def lists_of(row_ptr, cols):
    """The per-row lists of a (row_ptr, cols) pair, as sparse_attention_blocks takes them."""
    return [cols[row_ptr[i]:row_ptr[i + 1]] for i in range(len(row_ptr) - 1)]


def lift_mask(mask, perm, valid, block, n):
    """M^_uv = M_ij for u in R_i, v in R_j, over ORIGINAL token indices; [n, n] uint8."""
    region = np.empty(n, dtype=np.int64)
    for i in range(len(valid)):
        region[perm[i * block:i * block + valid[i]]] = i
    return mask[np.ix_(region, region)]


# ----------------------------------------------------------------------------
# attention
# ----------------------------------------------------------------------------
def full_attention(Q64, K64, V64):
    """Definition 3.1."""
    d = Q64.shape[1]
    return softmax_rows(Q64 @ K64.T / math.sqrt(d)) @ V64


def sparse_attention_dense(Q64, K64, V64, Mhat):
    """SparseAttn with the lifted mask on the full n x n logits (original order).

    Entries with M^ = 0 are excluded (logit -inf).  Only for small n.
    """
    d = Q64.shape[1]
    S = Q64 @ K64.T / math.sqrt(d)
    S = np.where(Mhat.astype(bool), S, -np.inf)
    return softmax_rows(S) @ V64


def sparse_attention_blocks(Qp64, Kp64, Vp64, idx, valid, block, rows=None, want_lse=False):
    """The same SparseAttn evaluated block by block on the reordered tensors.

    For query block i the keys are the valid slots of the blocks in idx[i]; pad query
    slots produce 0.  ``rows`` restricts the computation to those query blocks (the
    others stay 0).  Returns Op [n_pad, d] (and the natural-log LSE [n_pad]).
    """
    g = len(valid)
    d = Qp64.shape[1]
    Op = np.zeros_like(Qp64)
    lse = np.zeros(Qp64.shape[0], dtype=np.float64)
    scale = 1.0 / math.sqrt(d)
    for i in (range(g) if rows is None else rows):
        keys = np.concatenate([np.arange(j * block, j * block + valid[j]) for j in idx[i]])
        q = Qp64[i * block:i * block + valid[i]]
        S = (q @ Kp64[keys].T) * scale
        m = S.max(axis=1, keepdims=True)
        e = np.exp(S - m)
        z = e.sum(axis=1, keepdims=True)
        Op[i * block:i * block + valid[i]] = (e / z) @ Vp64[keys]
        lse[i * block:i * block + valid[i]] = (m + np.log(z))[:, 0]
    return (Op, lse) if want_lse else Op


# ----------------------------------------------------------------------------
# the whole path for one head
# ----------------------------------------------------------------------------
def forward_head(Q, K, V, dtype, T, fh, fw, ph, pw, sparsity=0.0, keep_blocks=0, rows=None, whole_map=False,
                 max_pool=False):
    """pool -> draft logits (canonical float32) -> top-k -> reorder -> sparse attention
    -> restore, for one head.  Q, K, V are stored [N, d] arrays (float32 values or bf16
    bit patterns).  Returns a dict with every intermediate.  ``rows`` as above (the
    restored output is then only meaningful for tokens of those query blocks).
    ``whole_map``: the threshold selection over the whole map instead of k per row; the
    result then carries row_ptr / cols, and idx is the list of per-row lists."""
    dims = derive_dims(T, fh, fw, ph, pw, sparsity, keep_blocks)
    block, n, k = dims["block"], dims["n"], dims["k"]
    perm, valid = reorder_index(T, fh, fw, ph, pw)
    inv = restore_index(perm, n)
    q32, k32 = widen_f32(Q, dtype), widen_f32(K, dtype)
    pool = pool_max_f32 if max_pool else pool_canonical_f32
    qp32 = pool(q32, perm, valid, block)
    kp32 = pool(k32, perm, valid, block)
    L32 = draft_logits_canonical_f32(qp32, kp32)
    row_ptr = cols = None
    if whole_map:
        row_ptr, cols, mask = select_blocks_global(L32, global_budget(dims["g"], sparsity, keep_blocks))
        idx = lists_of(row_ptr, cols)
    else:
        idx, mask = select_blocks(L32, k)
    Qp = permute(widen_f64(Q, dtype), perm)
    Kp = permute(widen_f64(K, dtype), perm)
    Vp = permute(widen_f64(V, dtype), perm)
    Op = sparse_attention_blocks(Qp, Kp, Vp, idx, valid, block, rows=rows)
    O = restore(Op, inv)
    return dict(dims=dims, perm=perm, inv=inv, valid=valid, q_pool=qp32, k_pool=kp32,
                logits=L32, idx=idx, mask=mask, row_ptr=row_ptr, cols=cols, Op=Op, O=O)
