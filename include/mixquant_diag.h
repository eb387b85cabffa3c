/*
 * mixquant_diag.h -- diagnostics exported by libmixquant next to the C ABI of mixquant.h.
 * Nothing here is part of the method; the benchmark uses it to state a measured roof beside the
 * published peak.
 */
#ifndef MIXQUANT_DIAG_H
#define MIXQUANT_DIAG_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueue a loop of `iters` x 8 independent FP16 MFMAs
 * (32x32x16) per wave on pseudo-random register operands, one wave per SIMD on 256 compute
 * units, with no memory traffic.  Timing it gives the matrix rate the chip sustains under its
 * power management for realistic operand toggling, the measured roof quoted beside the
 * published peak.  scratch_dev: at least one float of device memory (practically never
 * written).  *flop_out (host pointer, may be NULL) receives the flop count of the launch.
 * 1 <= iters <= 2^20.
 */
int mq_mfma_probe(float *scratch_dev, int iters, void *stream, double *flop_out);

#ifdef __cplusplus
}
#endif
#endif /* MIXQUANT_DIAG_H */
