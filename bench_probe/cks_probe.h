/*
 * cks_probe.h -- measurement probes used by bench.py (bench_probe/libcks_probe.so); not part of the
 * operators' library, its headers or its source tree.
 *
 * The operators of cks.h are bound by the fp32 matrix cores.  The published peak (157.3 TFLOP/s) assumes
 * every matrix instruction issues back to back at 2.4 GHz; what the chip sustains depends on the operand
 * values (constant operands run faster than varying ones) and on the clock under load.  These probes
 * measure both, so that the benchmark can state the achieved rate against the published AND the
 * sustained peak.
 *
 * All pointers are DEVICE pointers, `stream` is a hipStream_t (NULL = default stream), calls are
 * asynchronous.  Return 0 on success, -2 on bad arguments, -4 if the launch failed.  The caller times
 * the launches itself.
 */
#ifndef CKS_PROBE_H
#define CKS_PROBE_H

#ifdef __cplusplus
extern "C" {
#endif

/* `blocks` workgroups of 4 waves; each wave issues iters * 8 v_mfma_f32_32x32x2_f32 (4096 FLOPs each) on
 * two accumulators with operands held in registers.  random != 0: operands differ per lane, else all 1.0.
 * out: at least 256 floats, never written in practice. */
int cks_probe_mfma_registers(float *out, int blocks, int iters, int random, void *stream);

/* The K loop of the general kernels without global memory: `blocks` workgroups of 4 waves, each wave
 * issues items * chunks * 16 MFMAs fed by 16-byte LDS fragment reads, one workgroup barrier per chunk.
 * chunks must be even.  out: at least 256 floats. */
int cks_probe_mfma_lds(float *out, int blocks, int chunks, int items, int random, void *stream);

/* One wave writes n pairs (100 MHz wall-clock count, shader-clock count) to buf[2n], pausing `sleeps`
 * sleep instructions (about 3.4 us each) between samples; launched on a second stream it observes the
 * shader clock while other kernels run. */
int cks_probe_clock_samples(long long *buf, int n, int sleeps, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CKS_PROBE_H */
