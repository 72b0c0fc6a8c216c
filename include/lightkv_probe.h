/*
 * lightkv_probe.h -- two measurement kernels that state what the chip can deliver to the dense contractions of the
 * LightKV step (the feature divergence of Eq. "similarity" on large windows), used by bench.py --pass ceilings only.
 * They compute nothing of the method; they live in a library of their own (liblightkv_probe.so).
 *
 * Every function returns 0 on success, a hipError_t value otherwise; pointers are device memory unless named h_*;
 * work is enqueued on `stream` and the call waits for it (these are timing calls).
 */
#ifndef LIGHTKV_PROBE_H
#define LIGHTKV_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Operand delivery of a tiled A x B^T contraction with nothing else going on: every workgroup issues exactly the
 * global loads the tiled FD kernels issue for a tile x tile output tile -- bipartite (pairwise == 0: rows 2i of X are
 * the A rows, rows 2i+1 the B rows) or every row against every row (pairwise != 0) --, `piece_bytes` (128, 256 or 512)
 * per row and k-step, two k-steps in flight, the hidden axis cut into `splits` ranges that go to different workgroups;
 * the loaded values are only xor-ed together.  The calls allocate a few bytes of device memory and synchronise.
 *   X [n_rows, row_bytes] bf16 rows, row stride row_bytes; tile in {96, 128, 160, 192}
 *   h_us_out: average kernel time in microseconds over `iters` launches (HIP events on `stream`)
 *   h_bytes_out: bytes all workgroups together load per launch
 */
int lightkv_probe_operand_delivery(const void *X, int32_t n_rows, int32_t row_bytes, int32_t pairwise, int32_t tile,
                                   int32_t splits, int32_t piece_bytes, int32_t iters, float *h_us_out,
                                   double *h_bytes_out, void *stream);

/*
 * A bare loop of independent v_mfma_f32_32x32x16_bf16 (nine accumulators per wave, three operand fragments per side,
 * one wave per SIMD, n_workgroups workgroups of 256 threads).  operands: device, at least n_workgroups * 6 * 256 * 16
 * bytes of bf16 data -- what the fragments hold decides the clocks the chip sustains (constant vs. random operands).
 *   h_us_out: average kernel time; flops per launch = n_workgroups * 4 * 9 * mfma_per_acc * 32768
 */
int lightkv_probe_mfma(const void *operands, int32_t n_workgroups, int32_t mfma_per_acc, int32_t iters,
                       float *h_us_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LIGHTKV_PROBE_H */
