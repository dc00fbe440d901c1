/*
 * da.h - C ABI of the MI355X (gfx950) DraftAttention hot path.
 *
 * The path replaces full 3D attention in one attention module of a video diffusion
 * transformer (paper: arxiv 2505.14708, Section 3).  Per (batch, head):
 *
 *   pool Q,K inside each latent frame      Definition 3.2 (average pooling equations)
 *   draft map  softmax(Q~ K~^T / sqrt(d))  Definition 3.2 (draft attention map equation)
 *   keep the top k key blocks per row      "Guided Sparsity via Draft Attention"
 *     (or the top ceil(r g^2) of the map   Section 3.2.2, "Error from Sparsity Mask": the *_global and *_lists calls)
 *   reorder Q,K,V so a patch is a block    Algorithm 1, Section 3.3 "Execution"
 *   block-sparse attention                 SparseAttn equation, Section 3.1
 *   restore the order of O                 Algorithm 2, Section 3.3 "Restoration"
 *
 * Conventions common to every call
 *   - Tensors Q, K, V, O are [B, H, N, d], d fastest, contiguous, N = T*fh*fw and the token
 *     index is n = t*fh*fw + y*fw + x (the idx of Algorithm 1).  dtype DA_BF16 stores
 *     bfloat16, DA_F32 stores float.
 *   - A frame is cut into gh x gw = ceil(fh/ph) x ceil(fw/pw) patches anchored at (0,0);
 *     g = T*gh*gw blocks in (frame, patch row, patch column) order; block = ph*pw slots;
 *     n_pad = g*block.  A block holds its valid tokens in (row, column) raster order
 *     first and pad slots at its tail (Section 4.1 only says "appropriate padding").
 *   - Unless a parameter says "host", every pointer is a DEVICE pointer owned by the
 *     caller; the library neither allocates, frees nor keeps it.  Device pointers must be
 *     16-byte aligned.  Outputs must not alias inputs.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: no synchronisation, no host read-back, no allocation.
 *   - Return value: DA_OK (0) or a negative da_status.  On error nothing was launched,
 *     except DA_ERR_HIP, which reports a failed launch.  No global mutable state (but for the
 *     counter da_wait_failures reads); calls on different streams may run concurrently if their
 *     buffers are disjoint.
 *   - NaN/Inf in the inputs give unspecified values but never a fault.
 */
#ifndef DA_H
#define DA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { DA_F32 = 0, DA_BF16 = 1 };
/* How a region is pooled for the draft map: the mean (Definition 3.2), or the maximum (the other downsampling kernel
 * of the ablation, Section 4.3: per channel the largest value among the region's valid tokens). */
enum { DA_POOL_AVG = 0, DA_POOL_MAX = 1 };

typedef enum da_status {
  DA_OK = 0,
  DA_ERR_NULL = -1,        /* a required pointer is NULL */
  DA_ERR_DIM = -2,         /* a size is not positive, a ratio is outside [0,1), or a product overflows */
  DA_ERR_UNSUPPORTED = -3, /* valid, but no kernel: see da_sparse_attn */
  DA_ERR_WORKSPACE = -4,   /* ws_bytes is smaller than da_workspace_size() */
  DA_ERR_ALIGN = -5,       /* a device pointer is not 16-byte aligned */
  DA_ERR_HIP = -6,         /* the HIP runtime refused a launch */
  DA_ERR_SCRATCH = -7      /* the problem needs more scratch than the library's built-in buffer holds */
} da_status;

/* The problem statement of Definitions 3.1/3.2 and the inputs of Algorithm 1 (host struct). */
typedef struct da_problem {
  int32_t B, H;        /* batch, heads */
  int32_t T, fh, fw;   /* latent frames, frame height and width in tokens: Algorithm 1's F, H, W */
  int32_t d;           /* head dimension */
  int32_t ph, pw;      /* pooling window == stride: Algorithm 1's h, w */
  int32_t dtype;       /* DA_F32 or DA_BF16: storage type of Q, K, V, O and their reordered copies */
  int32_t keep_blocks; /* > 0: k given explicitly (clamped to g), `sparsity` ignored; 0: use `sparsity` */
  double  sparsity;    /* fraction of key blocks dropped per query block, in [0,1); the paper's r = 1 - sparsity */
  int32_t pool;        /* DA_POOL_AVG (0) or DA_POOL_MAX: what q_pool and k_pool hold, hence what the draft map ranks */
  int32_t reserved;    /* 0 */
} da_problem;

typedef struct da_dims {
  int32_t gh, gw;      /* patches per frame along y and x */
  int32_t g;           /* blocks (regions R_i of Definition 3.2) per head */
  int32_t block;       /* slots per block, ph*pw */
  int32_t k;           /* key blocks kept per query block: g - floor(sparsity*g + 1e-6), in [1,g] */
  int32_t reserved;
  int64_t n;           /* T*fh*fw */
  int64_t n_pad;       /* g*block */
} da_dims;

/* Layouts written by da_permute. */
enum {
  DA_REORDER_ROWS = 0, /* X [B,H,N,d] -> Xp [B,H,n_pad,d]; Xp[slot] = X[pi[slot]], zero rows in pad slots */
  DA_REORDER_VT = 1,   /* X [B,H,N,d] -> Xt [B,H,g,d,block]; Xt[i][c][s] = X[pi[i*block+s]][c], zeros in pad slots:
                          the reordered tensor with every block stored transposed (what da_sparse_attn wants for V
                          with DA_F32) */
  DA_RESTORE = 2,      /* Xp [B,H,n_pad,d] -> X [B,H,N,d]; X[n] = Xp[pi^-1[n]] */
  DA_REORDER_VOP = 3   /* X [B,H,N,d] -> Xo [B,H,g,block*d]: the transposed block cut into the 16-byte operands of the
                          bf16 matrix instructions, each operand group of 64 stored contiguously (what da_sparse_attn
                          wants for V with DA_BF16).  Only for DA_BF16, block a multiple of 64 and d a multiple of 32.
                          The reordered sequence is cut into sub-blocks of 64 slots; with nd = d/32, 16-byte unit
                          ((t*nd + dt)*64 + hh*32 + r) of sub-block b holds, for e = 0..7,
                          X[pi[b*64 + 16t + 8hh + e]][32dt + r]   (t < 4, dt < nd, hh < 2, r < 32), zeros in pad
                          slots */
};

/* Host only, pure.  Sizes that follow from the problem (see da_dims). */
int da_derive(const da_problem* p, da_dims* out /* host */);

/* Host only, pure.  Bytes of scratch da_forward needs for this problem. */
int da_workspace_size(const da_problem* p, size_t* bytes /* host */);

/*
 * Algorithm 1 (reorder index) and Algorithm 2 (restore index) as arrays, for callers that
 * want them; the other entry points compute the index arithmetic on the fly and do not
 * read these.  perm[n_pad] int32: original token at each slot, -1 in pad slots.
 * inv[n] int32: slot of each original token.  valid[g] int32: real tokens per block.
 * Any of the three may be NULL.  Only T, fh, fw, ph, pw of the problem are used.
 */
int da_build_perm(const da_problem* p, int32_t* perm, int32_t* inv, int32_t* valid, void* stream);

/*
 * Definition 3.2.  From Q and K [B,H,N,d] compute
 *   q_pool, k_pool [B,H,g,d] float : mean over the valid tokens of each block, float32,
 *       summed in slot order (acc = acc + x, one rounding per add) and divided once by
 *       the valid count (DA_POOL_MAX: their maximum instead, exact);
 *   logits [B,H,g,g] float : Q~ K~^T / sqrt(d) in float32 with the fixed order
 *       acc = fma(q[c], k[c], acc) for c = 0..d-1 (IEEE fused multiply-add, one rounding per term),
 *       then one multiply by float(1/sqrt(d));
 *   draft  [B,H,g,g] float : row softmax of logits (the draft attention map).
 * q_pool and k_pool are required; logits and draft may each be NULL (then not produced).
 * Any window ph, pw >= 1 and any d that is a multiple of 8 (bf16) or 4 (f32) is accepted.
 */
int da_draft_map(const da_problem* p, const void* Q, const void* K, float* q_pool, float* k_pool,
                 float* logits, float* draft, void* stream);

/*
 * Guided sparsity.  For every row of scores [B,H,g,g] (float) keep the k = da_dims.k
 * largest entries; equal values are kept lowest column first; -0 equals +0; NaN ranks
 * below every number.  idx [B,H,g,k] int32 receives the kept columns in ascending order.
 * mask [B,H,g,g] uint8 (may be NULL) receives M_ij in {0,1}.  The order is that of the
 * draft map whether scores holds logits or their row softmax.
 */
int da_select_blocks(const da_problem* p, const float* scores, int32_t* idx, uint8_t* mask, void* stream);

/* Reordering by pi of Algorithm 1 / restoring by pi^-1 of Algorithm 2; `mode` is one of
 * DA_REORDER_ROWS, DA_REORDER_VT, DA_RESTORE, DA_REORDER_VOP (layouts above).  Pure data movement. */
int da_permute(const da_problem* p, const void* X, void* Y, int mode, void* stream);

/*
 * SparseAttn on reordered tensors.  Qp, Kp [B,H,n_pad,d] (DA_REORDER_ROWS), Vt the reordered V
 * in the layout of its dtype (DA_REORDER_VOP for DA_BF16, DA_REORDER_VT for DA_F32), idx [B,H,g,k] int32 with entries in [0,g) (any order,
 * no repeats).  For query block i: Op[i*block+u] = sum_v softmax_v(Qp[u].Kp[v]/sqrt(d)) V[v]
 * over the valid slots v of the blocks in idx[i]; dropped blocks and pad keys get
 * probability 0.  Op [B,H,n_pad,d] in the problem's dtype; rows of pad query slots are
 * written with unspecified finite values.  lse [B,H,n_pad] float (may be NULL) receives the
 * natural-log normaliser of each row.
 * Supported: DA_BF16 with d = 128 and block = 64 or 128 (8x8 or 8x16 patches, say); DA_F32 with
 * d = 64 or 128 and block = 64; anything else returns DA_ERR_UNSUPPORTED.  bf16 uses bf16 MFMA with float32 accumulation and
 * softmax (and bf16 probabilities); f32 uses float32 arithmetic throughout.
 * The bf16 kernel leaves out, tile by tile (32 queries x 64 keys), keys whose probability is
 * negligible: a tile is dropped when each of its scores is so far below the best score its query
 * has met so far that everything dropped from a row adds up to less than 2^-14 of the row's largest
 * term (the cut is log2(block * k) + 14 powers of two).  The result differs from the full sum by less
 * than a bf16 rounding of the output; how much work is saved depends on how peaked the attention is
 * (nothing is dropped when all scores of a row are within that range of each other).
 * The bf16 kernel keeps the block lists of four query blocks (two when block = 128) in LDS, which
 * bounds the problem: roughly g/2 + 4*min(g, 4k) bytes must fit in 32 KB (g up to about 7000 with
 * nothing dropped, far more when k << g), and g * block / 64 < 2^22; larger problems return DA_ERR_UNSUPPORTED.  Its waits for tiles are
 * bounded; should one ever run out (no valid input makes it), the rows concerned are written as NaN.
 * Lists that are not what is asked for above (entries outside [0,g), repeats) give unspecified results but no access
 * outside the arrays: an entry that is no block number is left out.
 */
int da_sparse_attn(const da_problem* p, const void* Qp, const void* Kp, const void* Vt,
                   const int32_t* idx, void* Op, float* lse, void* stream);

/*
 * da_sparse_attn with two extras (SparseAttn equation, Section 3.1; Algorithms 1 and 2 by addressing).
 * original_order = 1 (DA_BF16 only): Q and O are the caller's [B,H,N,d] tensors in the ORIGINAL token order; the
 *   kernel reads each query row from, and writes each output row to, its original place, which is what da_forward
 *   does (Kp and Vt are still the reordered tensors; lse, if given, stays in slot order).  0: as da_sparse_attn.
 * tile_counts (DEVICE, two uint64, may be NULL; DA_BF16 only): the kernel ADDS to [0] the number of tiles
 *   (32 queries x 64 keys) its waves went through and to [1] the number of those whose exponentials and second
 *   product were carried out (the others fell to the drop rule described above).  The caller clears it.  Each tile
 *   is 16 matrix instructions for the first product and, if carried out, 16 for the second.
 */
int da_sparse_attn_ex(const da_problem* p, const void* Q, const void* Kp, const void* Vt, const int32_t* idx, void* O,
                      float* lse, int original_order, uint64_t* tile_counts, void* stream);

/*
 * Host call, synchronises the current device.  count (host) receives the number of wavefronts of the bf16 attention
 * kernel whose bounded wait for a key tile ran out (their rows were written as NaN) since the library was loaded,
 * on the current device.  No valid input makes that happen; a caller that wants to be sure checks for 0.
 */
int da_wait_failures(uint64_t* count /* host */);

/*
 * The whole path: O = restore(SparseAttn(reorder(Q,K,V), top-k(draft logits))).
 * Q, K, V, O [B,H,N,d].  idx_out [B,H,g,k] int32 (may be NULL) receives the kept blocks.
 * ws/ws_bytes: scratch of at least da_workspace_size() bytes, 256-byte aligned.
 * Same support matrix as da_sparse_attn.  The result is that of the separate calls; the launches
 * are fewer: K is reordered by the pooling pass, and for bf16 Q and O are never copied (the
 * attention kernel reads query rows from, and writes output rows to, their places in the original
 * order, which is Algorithm 1 for Q and Algorithm 2 for O done by addressing).
 * With every block kept (k = g: sparsity 0, the setting of the denoising steps that Section 4.1 leaves dense)
 * nothing is ranked: pooling, draft logits and selection are left out, the lists are 0 .. g-1, and the result is
 * full attention (Definition 3.1).  The same holds for da_forward_ex, and for da_forward_global with a budget of
 * g*g entries.
 */
int da_forward(const da_problem* p, const void* Q, const void* K, const void* V, void* O,
               int32_t* idx_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Where the rows of a caller's [B, H, rows, d] tensor live, for tensors that are not contiguous in that order (the
 * views of a fused [B, N, 3, H, d] projection, say): elements between consecutive batches, heads and rows.  A row
 * of d elements is contiguous; every stride is a multiple of 16 bytes and stride_n >= d.
 */
typedef struct da_layout {
  int64_t stride_b, stride_h, stride_n;
} da_layout;

/*
 * da_forward for other layouts of Q, K, V (`in`, one layout for the three) and O (`out`); NULL means contiguous
 * [B, H, rows, d].  reordered = 0: rows are the N tokens in the original order, as in da_forward.  reordered = 1:
 * the caller keeps its activations in the order of Algorithm 1 from layer to layer (Section 3.3's reordering is a
 * fixed permutation of the tokens, so it can be done once per model instead of once per attention): rows are the
 * n_pad slots, pad rows of Q, K, V must be zero, O's pad rows are left untouched (bf16) or unspecified, and a
 * contiguous K is used where it is.  Same support matrix, workspace and result as da_forward.
 */
int da_forward_ex(const da_problem* p, const da_layout* in, const da_layout* out, int reordered, const void* Q,
                  const void* K, const void* V, void* O, int32_t* idx_out, void* ws, size_t ws_bytes, void* stream);

/*
 * The whole-map form of the guided sparsity (Section 3.2.2, "Error from Sparsity Mask"): the threshold t is the
 * ceil(r g^2)-th largest score of a head's g x g map and M_ij = 1 where the score reaches t, so a row keeps as many
 * key blocks as it has scores above the threshold.  Readings: r = 1 - sparsity and the budget is
 * g^2 - floor(sparsity g^2 + 1e-6) entries (keep_blocks > 0: keep_blocks * g, the same total as that many per row);
 * exactly that many are kept: scores equal to t are taken in row-major order until the budget is used up (-0 equals
 * +0, NaN ranks below every number); a row that the threshold leaves empty keeps its best column (the lowest one
 * on ties), since its queries' attention is otherwise undefined.
 */
typedef struct da_global_dims {
  int64_t budget;     /* entries of one head's map kept by the threshold */
  int64_t cap;        /* entries to allocate per (batch, head) for the lists: budget + g rounded up to a multiple of 4 */
  size_t select_ws;   /* bytes of scratch da_select_blocks_global needs */
  size_t forward_ws;  /* bytes of scratch da_forward_global needs */
} da_global_dims;

/* Host only, pure.  DA_ERR_DIM when cap does not fit int32 or g^2 >= 2^32. */
int da_global_sizes(const da_problem* p, da_global_dims* out /* host */);

/*
 * Whole-map selection on scores [B,H,g,g] (float).  row_ptr [B,H,g+1] int32 receives, per head, the offsets of the
 * rows' lists (row_ptr[0] = 0, row_ptr[g] = entries kept, at most cap); cols [B,H,cap] int32 receives the kept
 * columns, row after row, ascending inside a row (entries past row_ptr[g] are left as they were).  mask [B,H,g,g]
 * uint8 may be NULL.  ws/ws_bytes: scratch of at least da_global_dims.select_ws bytes, 256-byte aligned.
 */
int da_select_blocks_global(const da_problem* p, const float* scores, int32_t* row_ptr, int32_t* cols, uint8_t* mask,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * da_select_blocks_global for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and result, minus ws: the scratch is a buffer of
 * DA_STATIC_SCRATCH_BYTES bytes built into the library (one per device, held until the process ends; its address
 * is looked up on the first call on a device).  The call allocates nothing and records no memset: everything that
 * must start at zero is cleared by a fill kernel on `stream`.  A problem whose da_global_dims.select_ws exceeds
 * DA_STATIC_SCRATCH_BYTES returns DA_ERR_SCRATCH and launches nothing.  All calls on one device share the one
 * buffer: calls that may overlap on a device (different streams, different threads) race; order them.
 */
#define DA_STATIC_SCRATCH_BYTES (32u << 20)
int da_select_blocks_global_static(const da_problem* p, const float* scores, int32_t* row_ptr, int32_t* cols,
                                   uint8_t* mask, void* stream);

/*
 * da_sparse_attn for lists of any length: query block i of head (b,h) attends the key blocks
 * cols[(b*H+h)*cap + row_ptr[(b*H+h)*(g+1) + i] .. row_ptr[.. + i + 1]) (entries in [0,g), any order, no repeats;
 * 0 <= row_ptr[..][i] <= row_ptr[..][i+1] <= cap; cap a multiple of 4).  A query block with an empty list gets zero
 * rows.  Everything else as da_sparse_attn (its k is not used; the cut of the bf16 drop rule goes by each row's own
 * number of keys); the bf16 kernel's LDS bound is that of k = g.  Offsets and entries that are not what is asked for
 * give unspecified results but no access outside the arrays (offsets are brought into [0,cap], entries outside [0,g)
 * are left out).
 */
int da_sparse_attn_lists(const da_problem* p, const void* Qp, const void* Kp, const void* Vt, const int32_t* row_ptr,
                         const int32_t* cols, int64_t cap, void* Op, float* lse, void* stream);

/*
 * da_forward with the whole-map selection.  row_ptr_out [B,H,g+1] and cols_out [B,H,cap] (both or neither may be
 * NULL) receive the kept blocks.  ws/ws_bytes: at least da_global_dims.forward_ws bytes, 256-byte aligned.
 */
int da_forward_global(const da_problem* p, const void* Q, const void* K, const void* V, void* O, int32_t* row_ptr_out,
                      int32_t* cols_out, void* ws, size_t ws_bytes, void* stream);

/* Static string for a da_status value (never NULL). */
const char* da_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DA_H */
