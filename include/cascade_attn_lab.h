/*
 * cascade_attn_lab.h -- measurement aids of the block-cascaded attention library.
 *
 * Not part of the method's boundary (that is cascade_attn.h): nothing here is a step of the path,
 * and a caller of the method needs none of it.  The benchmark and the tests use these two calls
 * to compare kernel variants inside one session and to read the attention kernel's rate against
 * what the matrix cores sustain on the same box.  Conventions as in cascade_attn.h, except that
 * ca_mfma_microbench synchronises.
 */
#ifndef CASCADE_ATTN_LAB_H
#define CASCADE_ATTN_LAB_H

#include "cascade_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Selects an attention kernel variant for experiments: 0 = default, 1 = no tail balancing (every
 * workgroup walks its whole KV range).  Unknown values are rejected with CA_EINVAL. */
int32_t ca_set_kernel_variant(ca_ctx* ctx, int32_t variant);

/* Measurement aid, not a step of the method: runs v_mfma_f32_32x32x16_bf16 back to back on every
 * CU (nothing else in the loop) and reports the sustained dense bf16 rate and the shader clock the
 * chip held meanwhile -- the practical ceiling to read cascade_attn_forward's TFLOP/s against.
 * data_kind 0: all-zero operands, 1: pseudo-random bf16 operands (more switching, lower clock).
 * trips: loop trips of 32 MFMAs per wave (100000 runs ~15 ms).  scratch_dev: device memory, at
 * least 16 bytes per CU, overwritten.  Synchronises the stream.  Either output may be NULL. */
int32_t ca_mfma_microbench(int32_t data_kind, int32_t trips, void* scratch_dev, size_t scratch_bytes,
                           void* hip_stream, double* tflops, double* clock_ghz);

#ifdef __cplusplus
}
#endif
#endif /* CASCADE_ATTN_LAB_H */
