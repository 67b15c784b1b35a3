/* Device-ceiling probes of liblexi_moe.so: measurement utilities for the roofline report, not part of the MoE
 * path.  The caller times the launches with HIP events on the stream it passes. */
#ifndef LEXI_PROBE_H
#define LEXI_PROBE_H
#include "lexi_moe.h"
#ifdef __cplusplus
extern "C" {
#endif

/*
 *   lexi_probe_mfma_bf16: `workgroups` workgroups of 4 waves, each wave issuing iters * 16 independent
 *     v_mfma_f32_32x32x16_bf16 (32768 flops each) on operand fragments read once from `operands` (device, at least
 *     40960 bytes of bf16 data: their bit patterns set the switching activity, hence the clock the chip sustains);
 *     flops = workgroups * 4 * iters * 16 * 32768.  sink: device, 1 KB, practically never written.
 *   lexi_probe_hbm_read: one streaming read of `bytes` bytes from src (device).  sink: device, 1 KB. */
lexi_status lexi_probe_mfma_bf16(const void* operands, void* sink, int32_t iters, int32_t workgroups, void* hip_stream);
lexi_status lexi_probe_hbm_read(const void* src, size_t bytes, void* sink, void* hip_stream);

/* Which schedule the down GEMM of lexi_moe_layer_forward(layer, T, k) into an independent output takes (a diagnostic
 * for tests and profiles; the choice never changes what is computed, only where the partial sums are added).
 *   which = 0: the routed experts' down GEMM; which = 1: the shared expert's.
 *   Returns 0 = weight-streaming schedule (decode-sized), 1 = tile schedule, 2 = tile schedule with the reduction cut
 *   in two (two partial planes, added by the combine), 3 = tile schedule storing the output rows directly (k = 1 and
 *   nothing else to add: no combine pass), 4 = a handful of tokens: weight streaming with the combine in the same
 *   launch; -1 = invalid arguments or no shared expert. */
int32_t lexi_moe_down_plan(const lexi_layer_t* layer, int32_t T, int32_t k, int32_t which);

#ifdef __cplusplus
}
#endif
#endif /* LEXI_PROBE_H */
