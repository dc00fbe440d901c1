/*
 * da_probe.h - three measuring sticks for bench.py: what the machine in front of us actually
 * sustains, next to its published peaks.  For callers that report a fraction of roofline and
 * want the measured ceiling beside the nominal one; not part of the attention path and not in
 * the product library: they are built into a library of their own (libdaprobe.so).
 */
#ifndef DA_PROBE_H
#define DA_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A loop of independent bf16 matrix instructions (v_mfma_f32_32x32x16_bf16, four accumulators per
 * wave, operands of random finite values) on every SIMD of the chip: `iters` trips of 16
 * instructions per wave.  sink: DEVICE buffer of at least 2^20 floats (receives checksums, so
 * that nothing is optimised away).  flop: HOST, receives the floating-point operations one
 * launch performs.  Only enqueues.  Returns 0, or a negative da_status value.
 */
int da_probe_mfma_bf16(int iters, float* sink, double* flop, void* stream);

/*
 * A plain copy of `bytes` bytes (a multiple of 16; both DEVICE pointers 16-byte aligned) with
 * non-temporal 16-byte loads and stores, 64 KB in a row per workgroup: bytes read + bytes written
 * = 2 * bytes.  Only enqueues.
 */
int da_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * A plain read of `bytes` bytes (a multiple of 16; DEVICE pointer, 16-byte aligned) with 16-byte loads, sixteen in
 * flight per lane, 128 KB in a row per workgroup; what was read is folded into checksums in sink (DEVICE, at least
 * 2^20 floats).  Only enqueues.
 */
int da_probe_read(const void* src, size_t bytes, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DA_PROBE_H */
