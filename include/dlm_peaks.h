/*
 * dlm_peaks.h -- C ABI of libdlm_peaks: three micro-benchmarks that measure what one MI355X (gfx950)
 * can actually sustain, so that kernel timings can be quoted against measured as well as nominal peaks.
 * A measuring instrument for the benchmark script; libdlm does not depend on it.
 *
 * All pointers are DEVICE pointers, 16-byte aligned; `bytes` must be a multiple of 16.  Calls enqueue on
 * `stream` (a hipStream_t, NULL = default) and return without synchronising; the caller times them with
 * events.  Return value: 0, or -1 for a bad argument, -4 when the launch failed.
 */
#ifndef DLM_PEAKS_H
#define DLM_PEAKS_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* dst[0 .. bytes) = src[0 .. bytes): 16 bytes per lane, 4 KB per workgroup.  nt bit 0: non-temporal loads,
 * bit 1: non-temporal stores.  Moves 2 * bytes through HBM. */
int dlm_peak_copy(const void *src, void *dst, size_t bytes, int nt, void *stream);

/* Reads src[0 .. bytes) once (16 bytes per lane, 16 KB per workgroup in 4 requests) and writes 4 bytes per
 * workgroup to sink (at least bytes / 16384 + 1 words).  nt != 0: non-temporal loads.  The ceiling of a kernel
 * that streams a large operand exactly once (W_vocab, a KV cache). */
int dlm_peak_read(const void *src, size_t bytes, int nt, uint32_t *sink, void *stream);

/* n_wg workgroups of 4 wavefronts, each wavefront issuing iters * 8 independent 32x32x16 bf16 MFMAs on
 * register operands (no memory traffic in the loop); sink receives one float per wavefront (n_wg * 4 floats).
 * FLOP = n_wg * 4 * iters * 8 * 32768; iters must be a multiple of 8.
 * operands == NULL: small constant operands (few bits toggle: the clock stays high; the silicon's ceiling).
 * operands != NULL: 16 * 64 * 16 bytes of bf16 values (e.g. N(0,1) draws), from which every lane takes eight
 *   different A and eight different B fragments, so consecutive MFMAs see different random operands: what the
 *   MFMA pipes sustain on realistic data, where the power limit lowers the clock.  This, not the nominal peak,
 *   bounds any bf16 contraction on such data. */
int dlm_peak_mfma(int n_wg, int iters, const void *operands, float *sink, void *stream);

/* Do matrix (MFMA) and vector-ALU instructions run side by side on a SIMD?  n_wg workgroups of 8 wavefronts (two per
 * SIMD); per iteration a "matrix" wavefront issues 4 independent 32x32x16 bf16 MFMAs, a "vector" wavefront 16
 * (fused multiply-add, exponential) pairs on 16 independent values.
 *   mode 0: all eight wavefronts matrix work;   mode 1: all eight vector work;
 *   mode 2: wavefronts 0-3 matrix, 4-7 vector (one of each kind per SIMD);
 *   mode 3: every wavefront both, each MFMA followed by four of the pairs in its own instruction stream.
 * If different wavefronts' MFMA and vector work overlapped, mode 2 would take the longer of half of mode 0 and half of
 * mode 1; if they exclude each other, the sum.  Mode 3 against modes 0 + 1 says the same for one wavefront's own stream.
 * sink: n_wg * 8 floats. */
int dlm_peak_overlap(int mode, int n_wg, int iters, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif
