/*
 * pshard_test -- entry points of libpshard.so that exist for tests and measurement only.
 *
 * None of these is part of the method's call surface (include/pshard.h): they expose the private
 * weight layout to host tests, let a GPU test look into the workspace or confirm an instruction's
 * operand layout, and time one kernel kind in isolation for the roofline report.
 */
#ifndef PSHARD_TEST_H
#define PSHARD_TEST_H

#include "pshard.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Pack a whole logical matrix (host scales fp16 [rows][K/32], host codes u8 [rows][K]) into
 * the private layout, rows in natural order; out: host, ps_packed_bytes(rows, K) bytes.
 * Layout: 16-row tiles, each a run of scale groups of up to 8 super-blocks (128 k); a
 * super-block is 64 lanes x 16 B, lane c*16+i = block 4*sb+c of row i, dword kk = weights
 * 8*kk..8*kk+7 of the block, weight t in nibble (t>>1) + 4*(t&1); after a group's
 * super-blocks come 64 lanes x 8 fp16 scales (lane c*16+i, entry s = block 4*(8g+s)+c). */
int32_t ps_pack_matrix(const uint16_t *scales, const uint8_t *codes, uint32_t rows, uint32_t K,
                       uint8_t *out);

/* ps_stack_set_decode_mode(st, PS_DECODE_MODE_OWN_RINV): mode 0, except that in a forward of 2..64
 * tokens the RMS factor of a hidden-state row always comes from a launch of its own; in modes 0 and
 * 1 the epilogue of an O or down matrix that one launch covers whole and that is summed from
 * split-K planes leaves the factor itself (same bits: the test of that claim is what this mode is
 * for). */
#define PS_DECODE_MODE_OWN_RINV 2

/* Time one kernel kind in isolation (measurement aid): every resident op of kind `kernel`
 * (PS_K_*) of a dense stack is launched back to back, `reps` passes after one warm-up pass,
 * between two events on the compute stream; *avg_launch_ms = elapsed / launches.  The
 * activations are whatever the workspace holds, the outputs go to the workspace.  Blocks. */
int32_t ps_stack_time_kernel(ps_stack *st, uint32_t kernel, uint32_t reps, double *avg_launch_ms,
                             uint32_t *launches);
/* device pointers into the workspace for inspection by tests (fp16 unless noted):
 * which = 0: QKV [M][qkv_w], 1: h [M][H], 2: s [M][I] or [M*top_k][I_e],
 * 3: route idx int32 [M][top_k], 4: route weights fp32 [M][top_k] */
int32_t ps_stack_debug_buffer(ps_stack *st, uint32_t which, void **dev_ptr, uint64_t *bytes);
/* Diagnostic: one v_mfma_f32_16x16x32_f16 with A = unit at (row pi, k pk) and B = unit at
 * (k pk, column pj); out_dev: device fp32 [64 lanes][4 registers] receives the accumulator.
 * Used by a GPU test to confirm the operand lane layout the GEMM kernel relies on.
 * pi, pj in 0..15, pk in 0..31; asynchronous on stream. */
int32_t ps_mfma_probe(int32_t pi, int32_t pk, int32_t pj, float *out_dev, void *stream);
/* Diagnostic: one LDS transpose read (ds_read_b64_tr_b16) by a wave over a table of the 16-bit numbers
 * 0 .. 2047 stored at their own index.  addr_dev: device uint32 [64], lane l's byte address into the
 * table (rounded down to a multiple of 8 and clamped inside it); out_dev: device uint16 [64][4], the
 * four numbers each lane received.  Used by a GPU test to confirm the lane layout the chunk-attention
 * kernels rely on for their V operand.  Asynchronous on stream. */
int32_t ps_lds_tr_probe(const uint32_t *addr_dev, uint16_t *out_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PSHARD_TEST_H */
