/*
 * Part of the CPU oracle (test infrastructure; see draft_attention.py): the float32 draft logits of Definition 3.2
 * (the draft attention map equation) in the one evaluation order that the kept-block decision is taken from.
 *
 *   acc = 0;  for c = 0 .. d-1:  acc = fma(q[c], k[c], acc)   (one rounding per term, IEEE fused multiply-add)
 *   L   = fl32(acc * scale)                                    (scale = fl32(1 / sqrt(d)), one more rounding)
 *
 * Plain loops, nothing blocked or reordered.  fmaf() is exact by definition; the target_clones attribute only lets the
 * compiler use the hardware instruction where the CPU has one (the default clone calls the C library's fmaf).
 * Build: gcc -O2 -ffp-contract=off -shared -fPIC draft_logits_fma.c -o _build/libdraftoracle.so -lm
 */
#include <math.h>

__attribute__((target_clones("fma", "default")))
void da_oracle_draft_logits_fma(const float* qp, const float* kp, float* out, long rows, long cols, long d, float scale) {
  for (long i = 0; i < rows; ++i) {
    for (long j = 0; j < cols; ++j) {
      float acc = 0.0f;
      for (long c = 0; c < d; ++c) acc = fmaf(qp[i * d + c], kp[j * d + c], acc);
      out[i * cols + j] = acc * scale;
    }
  }
}
