// Measurement helpers for the benchmark: what this machine actually sustains on the two resources
// the rooflines are quoted against, measured with the same launch and timing machinery as the
// kernels of the path.  Not part of the method.
//   probe_mfma_kernel    back-to-back v_mfma_f32_16x16x32_bf16 on 8 independent accumulators per
//                        wavefront, 8 wavefronts per SIMD: the practical dense bf16 matrix rate
//   probe_stream_kernel  every byte of a caller-provided buffer read once with 16-byte coalesced
//                        loads: the practical HBM read rate (use a buffer far larger than the caches)
//   probe_mix_kernel     the instruction mix of the softmax kernels, per loop step 16 MFMAs (four
//                        independent chains) and / or 16 x (fma, exp2, add) of vector work, four
//                        wavefronts per SIMD, in three launches: matrix work alone, vector work alone,
//                        both in one instruction stream.  How far "both" stays below the sum of the
//                        other two is how much the matrix cores and the vector ALU overlap.
//   probe_issue_kernel   what one instruction costs a SIMD's issue port: loops of independent fp32 fma's,
//                        of v_exp_f32, and of one MFMA followed by K independent fma's (K = 0, 2, 4), at
//                        four wavefronts per SIMD, timed over the whole chip; the benchmark reports them
//                        in units of one fma (4 cycles per wavefront instruction)
//   probe_fragment_kernel  the operand path of the attention kernels: every wavefront fetches 32 KiB
//                        blocks as 32 coalesced 1 KiB fragments (one 16-byte load per lane), from a
//                        2 MiB window that stays in L2, or from pseudo-random blocks of the whole buffer
//                        (which miss to the fabric)
#include "common.h"

namespace infllmv2 {

constexpr int kProbeMfmaIters = 2048, kProbeMfmaPerIter = 8, kProbeMfmaWgs = 256 * 8;

__global__ __launch_bounds__(256) void probe_mfma_kernel(float *__restrict__ sink, int iters, float seed) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(seed + 0.001f * (threadIdx.x & 15));
        b[i] = (__bf16)(seed * 0.5f + i);
    }
    f32x4 acc[kProbeMfmaPerIter];
#pragma unroll
    for (int i = 0; i < kProbeMfmaPerIter; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeMfmaPerIter; ++i) acc[i] = mfma16(a, b, acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeMfmaPerIter; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;      // keeps the loop alive, never true
}

__global__ __launch_bounds__(256) void probe_stream_kernel(const uint4 *__restrict__ buf, size_t n_u4,
                                                            uint32_t *__restrict__ sink) {
    uint32_t x = 0u;
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n_u4; i += stride) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = i + 256 * u < n_u4 ? buf[i + 256 * u] : uint4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 4; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (x == 0x9e3779b9u) sink[blockIdx.x * 256 + threadIdx.x] = x;      // never true for a zero-filled buffer
}

constexpr int kProbeMixIters = 4096, kProbeMixWgs = 256 * 4;

template <int kMode>   // 0: MFMA only, 1: vector ALU only, 2: both
__global__ __launch_bounds__(256) void probe_mix_kernel(float *__restrict__ sink, int iters, float c, float nm) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(c + 0.001f * (threadIdx.x & 15));
        b[i] = (__bf16)(c * 0.5f + i);
    }
    f32x4 acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    float x[16], s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = threadIdx.x * 0.01f + i;
    for (int it = 0; it < iters; ++it) {
        if (kMode != 1) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[u] = mfma16(a, b, acc[u]);
        }
        if (kMode != 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s += fast_exp2(__builtin_fmaf(x[i], c, nm));
                x[i] = __builtin_fmaf(x[i], 0.999f, 0.001f);      // a fourth vector instruction per element: keeps x live
            }
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) s += acc[u][0] + acc[u][1] + acc[u][2] + acc[u][3];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;      // keeps the loop alive, never true
}

constexpr int kProbeIssueIters = 8192, kProbeIssueWgs = 256;       // 1024 threads: four wavefronts per SIMD

// kMode 0: 8 fma per step, 1: 8 exp2 per step, 2 / 3 / 4: 4 x (one MFMA + 0 / 2 / 4 fma) per step; all
// instructions of a step independent of each other (written in assembly so that the compiler neither fuses
// nor reorders them)
template <int kMode>
__global__ __launch_bounds__(1024) void probe_issue_kernel(float *__restrict__ sink, int iters, float seed) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(seed + 0.001f * (threadIdx.x & 15));
        b[i] = (__bf16)(seed * 0.5f + i);
    }
    f32x4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = c0, c2 = c0, c3 = c0;
    float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1.f, x2 = x0 + 2.f, x3 = x0 + 3.f, x4 = x0 + 4.f, x5 = x0 + 5.f,
          x6 = x0 + 6.f, x7 = x0 + 7.f;
#define PROBE_M(c) "v_mfma_f32_16x16x32_bf16 %[" #c "], %[a], %[b], %[" #c "]\n"
#define PROBE_F(x, y) "v_fma_f32 %[" #x "], %[" #x "], %[" #x "], %[" #y "]\n"
#define PROBE_E(x) "v_exp_f32 %[" #x "], %[" #x "]\n"
#define PROBE_OPS                                                                                                  \
    : [c0] "+v"(c0), [c1] "+v"(c1), [c2] "+v"(c2), [c3] "+v"(c3), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2),      \
      [x3] "+v"(x3), [x4] "+v"(x4), [x5] "+v"(x5), [x6] "+v"(x6), [x7] "+v"(x7)                                    \
    : [a] "v"(a), [b] "v"(b)
    for (int it = 0; it < iters; ++it) {
        if (kMode == 0)
            asm volatile(PROBE_F(x0, x1) PROBE_F(x1, x2) PROBE_F(x2, x3) PROBE_F(x3, x4) PROBE_F(x4, x5) PROBE_F(x5, x6)
                             PROBE_F(x6, x7) PROBE_F(x7, x0) PROBE_OPS);
        if (kMode == 1)
            asm volatile(PROBE_E(x0) PROBE_E(x1) PROBE_E(x2) PROBE_E(x3) PROBE_E(x4) PROBE_E(x5) PROBE_E(x6) PROBE_E(x7)
                             PROBE_OPS);
        if (kMode == 2) asm volatile(PROBE_M(c0) PROBE_M(c1) PROBE_M(c2) PROBE_M(c3) PROBE_OPS);
        if (kMode == 3)
            asm volatile(PROBE_M(c0) PROBE_F(x0, x1) PROBE_F(x4, x5) PROBE_M(c1) PROBE_F(x1, x2) PROBE_F(x5, x6) PROBE_M(c2)
                             PROBE_F(x2, x3) PROBE_F(x6, x7) PROBE_M(c3) PROBE_F(x3, x0) PROBE_F(x7, x4) PROBE_OPS);
        if (kMode == 4)
            asm volatile(PROBE_M(c0) PROBE_F(x0, x1) PROBE_F(x4, x5) PROBE_F(x1, x2) PROBE_F(x5, x6) PROBE_M(c1)
                             PROBE_F(x2, x3) PROBE_F(x6, x7) PROBE_F(x3, x0) PROBE_F(x7, x4) PROBE_M(c2) PROBE_F(x0, x1)
                                 PROBE_F(x4, x5) PROBE_F(x1, x2) PROBE_F(x5, x6) PROBE_M(c3) PROBE_F(x2, x3) PROBE_F(x6, x7)
                                     PROBE_F(x3, x0) PROBE_F(x7, x4) PROBE_OPS);
    }
#undef PROBE_M
#undef PROBE_F
#undef PROBE_E
#undef PROBE_OPS
    const float s = c0[0] + c1[1] + c2[2] + c3[3] + x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;
    if (s == 12345.678f) sink[blockIdx.x * 1024 + threadIdx.x] = s;     // keeps the loop alive, never true
}

constexpr int kProbeFragWgs = 256 * 8, kProbeFragBlocks = 64;       // blocks of 32 KiB per wavefront

// kRandom false: block (wave id + i) mod 64 of a 2 MiB window; true: a pseudo-random block of the buffer
template <bool kRandom>
__global__ __launch_bounds__(256) void probe_fragment_kernel(const uint4 *__restrict__ buf, uint32_t n_blocks,
                                                              uint32_t *__restrict__ sink) {
    const uint32_t lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    uint32_t x = 0u, state = gw * 2654435761u + 12345u;
    for (int i = 0; i < kProbeFragBlocks; ++i) {
        state = state * 1664525u + 1013904223u;
        const uint32_t blk = kRandom ? (state >> 8) % n_blocks : (gw + i) & 63u;
        const uint4 *bp = buf + (size_t)blk * 2048 + lane;              // 2048 uint4 = 32 KiB
        uint4 v[32];
#pragma unroll
        for (int f = 0; f < 32; ++f) v[f] = bp[64 * f];
#pragma unroll
        for (int f = 0; f < 32; ++f) x ^= v[f].x ^ v[f].y ^ v[f].z ^ v[f].w;
    }
    if (x == 0x9e3779b9u) sink[blockIdx.x * 256 + threadIdx.x] = x;      // never true for a zero-filled buffer
}

// Launches the issue and fragment probes; work[] receives what each launch did: [0..4] instruction groups per
// SIMD of probe_issue_kernel<0..4> (a group = one fma, one exp2, or one MFMA with its 0 / 2 / 4 fma's),
// [5], [6] bytes fetched by probe_fragment_kernel<false / true>.
int launch_probes_detail(void *buf, size_t buf_bytes, double *work, hipStream_t stream) {
    static const char *const issue_names[5] = {"probe_issue_fma_kernel", "probe_issue_exp_kernel", "probe_issue_mfma_k0_kernel",
                                               "probe_issue_mfma_k2_kernel", "probe_issue_mfma_k4_kernel"};
    float *sink = reinterpret_cast<float *>(buf);
#define PROBE_ISSUE(MODE)                                                                                           \
    timing_begin(issue_names[MODE], stream);                                                                        \
    hipLaunchKernelGGL(probe_issue_kernel<MODE>, dim3(kProbeIssueWgs), dim3(1024), 0, stream, sink, kProbeIssueIters, \
                       1.0f);                                                                                       \
    timing_end(stream);                                                                                             \
    work[MODE] = 4.0 * kProbeIssueIters * (MODE < 2 ? 8 : 4);       /* four wavefronts per SIMD */
    PROBE_ISSUE(0)
    PROBE_ISSUE(1)
    PROBE_ISSUE(2)
    PROBE_ISSUE(3)
    PROBE_ISSUE(4)
#undef PROBE_ISSUE
    const uint32_t n_blocks = (uint32_t)(buf_bytes / 32768);
    timing_begin("probe_fragment_l2_kernel", stream);
    hipLaunchKernelGGL(probe_fragment_kernel<false>, dim3(kProbeFragWgs), dim3(256), 0, stream,
                       reinterpret_cast<const uint4 *>(buf), n_blocks, reinterpret_cast<uint32_t *>(buf));
    timing_end(stream);
    timing_begin("probe_fragment_random_kernel", stream);
    hipLaunchKernelGGL(probe_fragment_kernel<true>, dim3(kProbeFragWgs), dim3(256), 0, stream,
                       reinterpret_cast<const uint4 *>(buf), n_blocks, reinterpret_cast<uint32_t *>(buf));
    timing_end(stream);
    work[5] = work[6] = (double)kProbeFragWgs * 4 * kProbeFragBlocks * 32768.0;
    return (int)hipGetLastError();
}

int launch_probes(void *buf, size_t buf_bytes, double *mfma_flops, double *stream_bytes, hipStream_t stream) {
    // the first 4 MiB of the buffer double as the (never written) sink of both kernels
    const size_t n_u4 = buf_bytes / sizeof(uint4);
    timing_begin("probe_mfma_kernel", stream);
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeMfmaWgs), dim3(256), 0, stream, reinterpret_cast<float *>(buf),
                       kProbeMfmaIters, 1.0f);
    timing_end(stream);
    timing_begin("probe_stream_kernel", stream);
    hipLaunchKernelGGL(probe_stream_kernel, dim3(256 * 16), dim3(256), 0, stream, reinterpret_cast<const uint4 *>(buf),
                       n_u4, reinterpret_cast<uint32_t *>(buf));
    timing_end(stream);
    timing_begin("probe_mix_mfma_kernel", stream);
    hipLaunchKernelGGL(probe_mix_kernel<0>, dim3(kProbeMixWgs), dim3(256), 0, stream, reinterpret_cast<float *>(buf),
                       kProbeMixIters, 0.1f, -3.f);
    timing_end(stream);
    timing_begin("probe_mix_valu_kernel", stream);
    hipLaunchKernelGGL(probe_mix_kernel<1>, dim3(kProbeMixWgs), dim3(256), 0, stream, reinterpret_cast<float *>(buf),
                       kProbeMixIters, 0.1f, -3.f);
    timing_end(stream);
    timing_begin("probe_mix_both_kernel", stream);
    hipLaunchKernelGGL(probe_mix_kernel<2>, dim3(kProbeMixWgs), dim3(256), 0, stream, reinterpret_cast<float *>(buf),
                       kProbeMixIters, 0.1f, -3.f);
    timing_end(stream);
    *mfma_flops = (double)kProbeMfmaWgs * 4 * kProbeMfmaIters * kProbeMfmaPerIter * (2.0 * 16 * 16 * 32);
    *stream_bytes = (double)n_u4 * sizeof(uint4);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
