/*
 * sig_probe.h -- measurement anchors that ship with libsig.  They are not part of the
 * signature transform; callers are benchmarks and profiling runs that need (a) a copy kernel
 * of known size, to calibrate the HBM byte counters and to measure the achievable HBM rate, and
 * (b) an FMA loop of known flop count, to measure the achievable fp32 vector rate without packed
 * instructions (every translation unit of this library is built with packed fp32 switched off), and
 * (c) write-only kernels, plain and with the access pattern of the stream-mode kernels.
 * Same conventions as sig.h: DEVICE pointers, hipStream_t passed as void*, status codes of enum
 * sig_status, nothing synchronises.
 */
#ifndef SIG_PROBE_H
#define SIG_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dst[i] = src[i] for n_floats floats (n_floats % 4 == 0, both 16-byte aligned); reads and writes 4*n_floats bytes each. */
int sig_probe_copy(float *dst, const float *src, int64_t n_floats, void *hip_stream);

/*
 * Every lane of `waves` wavefronts (workgroups of 4) runs `iters` rounds of 16 fp32 FMAs arranged as
 * `ilp` independent dependency chains (1, 2, 4, 8 or 16) and stores one float to out[lane id]
 * (out: DEVICE, waves * 64 floats).  `lds_bytes` (0 .. 65536) of dynamic LDS are requested per
 * workgroup only to limit how many workgroups share a compute unit.
 * Flops = 2 * 16 * iters * waves * 64.
 */
int sig_probe_fma(float *out, int64_t waves, int64_t iters, int ilp, int lds_bytes, void *hip_stream);

/*
 * The instruction form of the signature kernels' inner loops: every lane keeps a 10 x 10 block of accumulators and
 * runs `iters` rounds of acc[a][b] += g[a] * v[b] (100 fp32 FMAs per round, each reading three vector registers:
 * the accumulator and two operands that change from instruction to instruction), which is what the sum of rank-1
 * updates of Eq. 3 compiles to.  The rate of this form, at the occupancy a kernel's register count allows, is the
 * ceiling of the fused kernels; it lies below the rate of sig_probe_fma, whose FMAs take one operand from a literal.
 * Same arguments as sig_probe_fma.  Flops = 2 * 100 * iters * waves * 64.
 */
int sig_probe_fma_outer(float *out, int64_t waves, int64_t iters, int lds_bytes, void *hip_stream);

/*
 * Write-only anchors for the stream-mode kernels, whose traffic is almost all stores.
 * streams == 1: a plain fill, dst[i] = 1 for n_floats floats, the grid sweeping memory front to back.
 * streams  > 1: `streams` sequential write cursors advancing together, one wavefront per cursor (the pattern of
 *   a stream-mode launch: every path's rows are a region of its own): dst is cut into `streams` equal regions of
 *   n_floats / streams floats (a multiple of 4), each written front to back by its own wavefront.
 * dst: DEVICE, 16-byte aligned, n_floats % (4 * streams) == 0.  Writes 4 * n_floats bytes.
 */
int sig_probe_write(float *dst, int64_t n_floats, int64_t streams, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
