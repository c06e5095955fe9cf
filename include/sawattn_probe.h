/*
 * sawattn_probe -- a measurement aid of the benchmark, not part of the attention path: the matrix rate an
 * MI355X sustains, next to which the attention kernel's rate is read.  C ABI of libsawattn_probe.so.
 */
#ifndef SAWATTN_PROBE_H
#define SAWATTN_PROBE_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * sawattn_mfma_probe -- launches one 8-wavefront workgroup per compute unit; each wavefront issues iters*16
 * v_mfma_f32_32x32x16_f16 on four independent accumulators.  No passage of the paper corresponds to it; the
 * paper reports throughput only (Sec. 4.2 / 4.3), and this gives the ceiling that throughput is read against.
 *
 *   sink       device, >= 512 floats; never written in practice (keeps the work alive).
 *   iters      > 0.
 *   mode       0: all operands zero (no switching in the multipliers: the datasheet condition);
 *              1: operands in registers with values distributed like attention inputs;
 *              2: as 1, with the A operands re-read from an LDS tile with the attention kernel's
 *                 K-operand pattern.  The chip is power limited: 1 and 2 run far below 0.
 *   hip_stream stream to launch on (NULL = default); returns without waiting.
 *   flops_out  host, optional: receives the flop count of the launch (2*32*32*16 per MFMA).
 * Returns 0, 1 (invalid argument) or 3 (the HIP runtime refused); text from sawattn_probe_last_error().
 */
int sawattn_mfma_probe(float* sink, int iters, int mode, void* hip_stream, double* flops_out);

/* Text of the last error raised on the calling thread ("" if none).  Static storage, never NULL. */
const char* sawattn_probe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SAWATTN_PROBE_H */
