/*
 * Measured ceilings of the GPU libswitchback runs on.  Measurement aids for the benchmark: no step of the SwitchBack
 * layer (arxiv 2304.13013) runs through these calls.  They answer "what do the matrix pipes and the memory system of
 * this GPU sustain for code that does nothing else", which is what a kernel's fraction of the published peak has to be
 * read against: the published matrix peaks assume a clock the GPU does not hold under load, and how far the clock
 * drops depends on the operand values (toggling bits draw power).
 *
 * Conventions as in switchback.h: device pointers owned by the caller, 16-byte aligned; calls only enqueue on
 * `stream`; nothing is allocated; status codes of sb_status.
 */
#ifndef SWITCHBACK_CEILINGS_H
#define SWITCHBACK_CEILINGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Which matrix instruction the loop issues: v_mfma_i32_32x32x32_i8, v_mfma_f32_32x32x16_bf16 or
 * v_mfma_f32_32x32x64_f8f6f4 (E4M3 x E4M3) -- the instructions of the library's three product kernels. */
typedef enum { SB_CEILING_I8 = 0, SB_CEILING_BF16 = 1, SB_CEILING_F8 = 2 } sb_ceiling_kind;

/* Register-resident matrix-instruction loop.  Every wave loads the operand fragment set of the product kernels (four
 * token-side and two weight-side fragments for each of two k-steps; a fragment is 16 bytes per lane, 32 for float8)
 * once from a_codes / b_codes (wave w starts at its own offset, wrapping around the buffers) and then issues the
 * sixteen products of the set `iters` times: no LDS, no memory traffic inside the loop.  The operand VALUES are the
 * caller's: zeros, random codes, or codes the library's quantizers produced from a workload.
 *   a_codes [a_bytes], b_codes [b_bytes]: device buffers, lengths multiples of one wave fragment (1024 bytes; 2048 for
 *   float8); workgroups x waves_per_workgroup (4 or 8) waves are launched; sink: device floats, one per lane launched
 *   (workgroups * waves_per_workgroup * 64), written once at the end; ops_out: optional HOST pointer that receives the
 *   number of operations (2 per multiply-add) the launch performs. */
int switchback_ceiling_mfma(int kind, const void *a_codes, size_t a_bytes, const void *b_codes, size_t b_bytes,
                            int workgroups, int waves_per_workgroup, int iters, float *sink, double *ops_out,
                            void *stream);

/* Plain device copy, 16 bytes per lane, every byte read once and written once (bytes % 16 == 0). */
int switchback_ceiling_copy(const void *src, void *dst, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SWITCHBACK_CEILINGS_H */
