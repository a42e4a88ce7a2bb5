/*
 * longlive_diag.h - diagnostics and tuning knobs of the MI355X (gfx950) LongLive library.
 *
 * Nothing in this header is part of the method: these calls exist to benchmark the library's own kernel variants
 * against each other and to measure what the GPU's matrix pipe sustains, so that the attention kernel's rate can be
 * read against the rate a pure stream of matrix instructions reaches on the same chip in the same run.
 * Conventions (status codes, device/host pointers, streams) are those of longlive.h.
 */
#ifndef LONGLIVE_DIAG_H
#define LONGLIVE_DIAG_H

#include "longlive.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Attention kernel variant: 0 = default for the shape, otherwise a variant id listed by
 * ll_attn_variant_name.  Process-wide tuning knob for benchmarking. */
ll_status ll_set_attn_variant(int variant);
const char* ll_attn_variant_name(int variant); /* NULL when `variant` does not exist */

/* Diagnostic, not part of the method: the dense bf16 MFMA rate this GPU sustains when every wave issues nothing
 * but 32x32x16 MFMAs (two waves per SIMD, `workgroups` workgroups of 8 waves, iters * 16 MFMAs per wave), and the
 * core clock it settles at while doing so.  random_operands != 0 fills the operand registers with random bf16
 * mantissas and signs, 0 with the constant 1.0: under a full matrix load the chip is power-limited and the clock
 * depends on how many operand bits toggle, so the two differ by about a third.  bench.py reports the attention
 * kernel's rate next to the random-operand figure.
 *   dev_scratch: device, at least workgroups * 2048 + 16 bytes, contents overwritten.
 *   The kernel runs twice on `stream` (the first run lets the clock settle, the second is timed with events);
 *   the call returns after the stream has finished.  tflops, clock_ghz: host. */
ll_status ll_probe_mfma_rate(void* dev_scratch, size_t scratch_bytes, int workgroups, int iters,
                             int random_operands, double* tflops, double* clock_ghz, void* stream);
/* The same loop with company: `per_mfma` (1 or 2) instructions of kind `companion` issued behind every MFMA, on
 * registers no MFMA touches: 0 none, 1 v_add_f32, 2 v_exp_f32, 3 v_cvt_pk_bf16_f32, 4 v_dot2c_f32_bf16,
 * 5 v_max3_f32, 6 ds_read_b128 (64 KB of LDS, conflict-free), 7 no companion but 16x16x32 MFMAs (twice as many,
 * the same flops).  The drop against companion 0 is what that instruction costs the matrix pipe in issue slots and,
 * with random operands, in power.  tflops counts the MFMA flops only.  Other arguments as above.
 * Companions 8 to 11 run fp8 MFMAs instead (32x32x64, E4M3 operands, four times the flops per instruction; per_mfma
 * is ignored): 8 alone, 9 with what the 8-bit attention kernel issues per MFMA (4 v_exp_f32, 4 v_add_f32,
 * 2 v_cvt_pk_fp8_f32, 2 v_max3_f32, 2 ds_read_b128), 10 with the vector part of that only, 11 with the LDS part only. */
ll_status ll_probe_mfma_mix(void* dev_scratch, size_t scratch_bytes, int workgroups, int iters, int random_operands,
                            int companion, int per_mfma, double* tflops, double* clock_ghz, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LONGLIVE_DIAG_H */
