/*
 * tca_diag.h - diagnostics of libtca.so.  Nothing here is a step of the method or
 * part of its boundary (tca.h); the benchmark uses these to report what the board
 * sustains and to compare kernel shapes.  The two switches are process-wide and
 * meant to be set before the calls they affect, from one thread.
 */
#ifndef TCA_DIAG_H
#define TCA_DIAG_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* tca_probe_mfma times a register-only loop of bf16 32x32x16 MFMAs that fills every SIMD
 * (`iters` x 16 MFMAs per wave) and reports the rate it reached and the shader clock it ran at
 * (cycle counter over the constant 100 MHz counter).  random_operands != 0 gives the operands
 * random signs and magnitudes, 0 makes them constants; the difference is the board's power
 * limit, which bounds what any MFMA kernel on real data can reach.  ws: device scratch of
 * tca_probe_workspace_bytes() bytes, 256-byte aligned.  Synchronises the stream.
 * Returns 0 or a negative TCA_ERR_* code. */
size_t tca_probe_workspace_bytes(void);
int tca_probe_mfma(int random_operands, int iters, double* tflops, double* shader_ghz,
                   void* ws, size_t ws_bytes, void* stream);

/* enable != 0: every later TCA_BF16 tca_prefill call leaves, in the first four uint64 of its
 * workspace, sums over the workgroups of its attention kernel (four atomic adds per workgroup):
 * elapsed shader-clock cycles; elapsed 100 MHz ticks (cycles / ticks / 10 is the average
 * shader clock in GHz); the cycles that passed before the first tile step; the 64-key tiles
 * walked.  Off by default: the kernel then records nothing. */
void tca_diag_prefill_clocks(int enable);

/* Workgroup shape of the bf16 prefill kernel: 0 = chosen by the size of the call (default);
 * 1 = 4 waves x 32 queries; 2 = 4 waves x 64 queries (one wave per SIMD, every LDS fragment
 * feeds two MFMAs); 3 = 8 waves x 32 queries.  All shapes compute the same result. */
int tca_diag_prefill_variant(int variant);

#ifdef __cplusplus
}
#endif
#endif /* TCA_DIAG_H */
