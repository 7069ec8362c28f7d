/*
 * Measurement entry points of libinfllmv2_bench.so, the bench-only build of the library: the same
 * kernels and entry points as libinfllmv2.so (include/infllmv2.h), plus per-kernel event timing around
 * every launch and the probe kernels that measure what the machine sustains.  Not part of the product
 * library, and unlike its entry points these SYNCHRONISE (infllmv2_timing_read waits for the recorded
 * launches) and keep process-wide state that is NOT thread-safe: one thread, one device, benchmarks only.
 */
#ifndef INFLLMV2_BENCH_H
#define INFLLMV2_BENCH_H

#include "infllmv2.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measured practical peaks for the benchmark's rooflines (not part of the method).  Launches
 * probe kernels on `stream`: a dense bf16 MFMA loop ("probe_mfma_kernel"), a read of every byte
 * of `buf` ("probe_stream_kernel"), and the instruction mix of a softmax kernel as matrix work
 * alone, vector work alone and both together ("probe_mix_mfma_kernel", "probe_mix_valu_kernel",
 * "probe_mix_both_kernel": the same loop count each, so their durations compare directly); the
 * durations are obtained like any other kernel's, through infllmv2_timing_enable /
 * infllmv2_timing_read.
 *   buf            in   DEVICE buffer, 256-byte aligned, at least 8 MiB, ZERO-FILLED by the caller
 *                       (it is only read; a size far above the cache sizes measures HBM)
 *   mfma_flops     out  HOST: floating-point operations the MFMA probe executes per launch
 *   stream_bytes   out  HOST: bytes the stream probe reads per launch
 */
int32_t infllmv2_probe_peaks(void *buf, size_t buf_bytes, double *mfma_flops, double *stream_bytes,
                             void *stream);

/*
 * Finer probes behind the bounds the design notes argue with; durations through infllmv2_timing_read.
 *   "probe_issue_fma_kernel", "probe_issue_exp_kernel", "probe_issue_mfma_k0 / k2 / k4_kernel": loops of
 *       independent instructions at four wavefronts per SIMD -- fp32 fma; v_exp_f32; one 16x16x32 bf16 MFMA
 *       followed by 0 / 2 / 4 fma's.  work[0..4] = instruction groups executed per SIMD (a group = one fma,
 *       one exp2, or one MFMA with its fma's): duration / work[i] is the issue cost of a group.
 *   "probe_fragment_l2_kernel", "probe_fragment_random_kernel": every wavefront fetches 32 KiB blocks as 32
 *       coalesced 1 KiB fragments, from a 2 MiB window (L2 hits) or from pseudo-random blocks of the whole
 *       buffer (misses).  work[5], work[6] = bytes fetched.
 *   buf    in   DEVICE buffer as for infllmv2_probe_peaks (zero-filled, only read)
 *   work   out  HOST array of 7 doubles
 */
int32_t infllmv2_probe_detail(void *buf, size_t buf_bytes, double *work, void *stream);

/*
 * Per-kernel timing for benchmarks (the measurement the roofline figures are built on).
 * While enabled, every kernel launched by the entry points above is bracketed by HIP events
 * recorded on the call's stream; at most 256 launches are kept between reads.  Process-wide
 * state, not thread-safe; leave it off in production (each launch costs two event records).
 *   infllmv2_timing_enable  enable != 0 creates the events on the current device on first use
 *                           and clears the log; 0 switches recording off.
 *   infllmv2_timing_read    waits for the recorded launches to finish, writes up to max_entries
 *                           (kernel name, milliseconds) pairs in launch order into the HOST
 *                           arrays names / ms, clears the log, and returns the count (>= 0) or
 *                           a negative status.
 */
int32_t infllmv2_timing_enable(int32_t enable);
int32_t infllmv2_timing_read(int32_t max_entries, const char **names, float *ms);

#ifdef __cplusplus
}
#endif
#endif /* INFLLMV2_BENCH_H */
