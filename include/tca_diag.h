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

/* How a TCA_BF16 tca_prefill call with these sizes spreads its work over the chip (host only, nothing is
 * launched): the kernel walks the (head, query tile) items head by head, a head's query tiles from the
 * last to the first, and XCD x takes the items [start_out[x], start_out[x + 1]).
 *   offs : host [Hs + 1], as for tca_prefill;  part : TCA_PART_ALL / _WINDOW / _GLOBAL;
 *   gather_free != 0 : the call would have Kg = Vg = NULL;  start_out : host int32 [9]
 * Returns the number of workgroups of the attention kernel, or -1 (not a bf16 call, head count not a
 * multiple of 8, invalid sizes). */
int64_t tca_diag_prefill_xcd_plan(const tca_params* prm, const int64_t* offs, int64_t q_pos0, int64_t n_queries,
                                  int part, int gather_free, int32_t* start_out);

#ifdef __cplusplus
}
#endif
#endif /* TCA_DIAG_H */
