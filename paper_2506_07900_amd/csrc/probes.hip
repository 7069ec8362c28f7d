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
