// Stage 1: mean-pool compression of the key cache into semantic-kernel representations
// (section 2.1.2, "Semantic Kernels": S_jh = K[jh*s : jh*s+p], representation Mean(S_jh)),
// and the decode-step cache append.  Both are pure HBM traffic: 16-byte coalesced rows.
#include "common.h"

namespace infllmv2 {

// One thread = 8 channels of one semantic kernel; 16 threads cover a 128-wide row, so a
// 256-thread workgroup produces 16 kernels.  The sum runs in fp64 in token order: for bf16
// inputs it is exact, so the result is the correctly rounded mean.
__global__ __launch_bounds__(256) void compress_keys_kernel(Dims dm, Tensor k, Tensor ck,
                                                             const int32_t *__restrict__ seqlens,
                                                             int32_t n_new_tokens) {
    const int b = blockIdx.z, h = blockIdx.y;
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int32_t n_c = num_kernels(L);
    int32_t first = 0;
    if (n_new_tokens > 0) first = num_kernels(L - n_new_tokens > 0 ? L - n_new_tokens : 0);
    const int c = (threadIdx.x & 15) * 8;
    const __bf16 *kb = k.ptr + b * k.sb + h * k.sh + c;
    __bf16 *ob = ck.ptr + b * ck.sb + h * ck.sh + c;
    for (int32_t jh = first + blockIdx.x * 16 + (threadIdx.x >> 4); jh < n_c; jh += gridDim.x * 16) {
        double acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.0;
        const __bf16 *row = kb + (int64_t)jh * kStride * k.st;
#pragma unroll 8
        for (int t = 0; t < kKernel; ++t) {
            bf16x8 x = load8(row + (int64_t)t * k.st);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (double)(float)x[e];
        }
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t lo = f64_to_bf16_rne(acc[2 * e] / (double)kKernel);
            uint32_t hi = f64_to_bf16_rne(acc[2 * e + 1] / (double)kKernel);
            w[e] = lo | (hi << 16);
        }
        uint4 o = {w[0], w[1], w[2], w[3]};
        *reinterpret_cast<uint4 *>(ob + (int64_t)jh * ck.st) = o;
    }
}

int launch_compress_keys(const Dims &dm, Tensor k, Tensor ck, const int32_t *seqlens,
                         int32_t n_new_tokens, hipStream_t stream) {
    int32_t per_seq = num_kernels(dm.max_seqlen);
    if (n_new_tokens > 0) {
        int32_t inc = n_new_tokens / kStride + 1;
        if (inc < per_seq) per_seq = inc;
    }
    if (per_seq <= 0 || dm.batch <= 0) return 0;
    dim3 grid((per_seq + 15) / 16, dm.Hkv, dm.batch);
    timing_begin("compress_keys_kernel", stream);
    hipLaunchKernelGGL(compress_keys_kernel, grid, dim3(256), 0, stream, dm, k, ck, seqlens,
                       n_new_tokens);
    timing_end(stream);
    return (int)hipGetLastError();
}

// Decode-step append: copy the new key / value rows of every (sequence, key-value head) to
// cache positions seqlens[b]-n_q .. seqlens[b]-1 (n_q = 1 in plain decode; the drafted tokens of a
// verification step otherwise).  One 16-lane group per row.  With kWithCk (n_q = 1 only) the same launch also
// writes the semantic-kernel representation that the new token completes (it ends kernel
// jh = (L-32)/16 when L >= 32 and L-32 is a multiple of 16): its 31 older rows come from the
// cache, the newest from k_new, summed in fp64 like compress_keys_kernel (exact for bf16 inputs).
template <bool kWithCk>
__global__ __launch_bounds__(256) void append_kv_kernel(Dims dm, Tensor k_new, Tensor v_new, Tensor k,
                                                         Tensor v, Tensor ck, const int32_t *__restrict__ seqlens) {
    const int row = blockIdx.x * 16 + (threadIdx.x >> 4);   // (b, h, new token) triple
    if (row >= dm.batch * dm.Hkv * dm.n_q) return;
    const int bh = row / dm.n_q, qi = row - bh * dm.n_q;
    const int b = bh / dm.Hkv, h = bh % dm.Hkv;
    const int32_t L = seqlens[b] - (dm.n_q - 1 - qi);       // cache rows up to and including this token
    if (L < 1 + qi || seqlens[b] > dm.max_seqlen) return;   // a sequence shorter than n_q is skipped as a whole
    const int c = (threadIdx.x & 15) * 8;
    const int64_t dst = (int64_t)(L - 1);
    const uint4 kn = *reinterpret_cast<const uint4 *>(k_new.ptr + b * k_new.sb + h * k_new.sh + qi * k_new.st + c);
    const __bf16 *kb = k.ptr + b * k.sb + h * k.sh + c;
    const bool closes = kWithCk && L >= kKernel && (L - kKernel) % kStride == 0;
    bf16x8 old[kKernel - 1];
    if (closes) {
#pragma unroll
        for (int t = 0; t < kKernel - 1; ++t) old[t] = load8(kb + (int64_t)(L - kKernel + t) * k.st);
    }
    *reinterpret_cast<uint4 *>(k.ptr + b * k.sb + h * k.sh + dst * k.st + c) = kn;
    *reinterpret_cast<uint4 *>(v.ptr + b * v.sb + h * v.sh + dst * v.st + c) =
        *reinterpret_cast<const uint4 *>(v_new.ptr + b * v_new.sb + h * v_new.sh + qi * v_new.st + c);
    if (closes) {
        const bf16x8 newest = __builtin_bit_cast(bf16x8, kn);
        double acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.0;
#pragma unroll
        for (int t = 0; t < kKernel - 1; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (double)(float)old[t][e];
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = f64_to_bf16_rne((acc[2 * e] + (double)(float)newest[2 * e]) / (double)kKernel);
            const uint32_t hi = f64_to_bf16_rne((acc[2 * e + 1] + (double)(float)newest[2 * e + 1]) / (double)kKernel);
            w[e] = lo | (hi << 16);
        }
        const int32_t jh = (L - kKernel) / kStride;
        *reinterpret_cast<uint4 *>(ck.ptr + b * ck.sb + h * ck.sh + (int64_t)jh * ck.st + c) =
            uint4{w[0], w[1], w[2], w[3]};
    }
}

// Verification-step append in one launch: workgroups 0 .. n_copy-1 of a (sequence, head) copy the
// n_q new rows into the caches, the others write the semantic kernels those rows complete, reading
// the rows that are new from k_new and the older ones from the cache (fp64 sum in token order, one
// rounding: the bits compress_keys_kernel produces once the rows are in the cache).
__global__ __launch_bounds__(256) void append_compress_kernel(Dims dm, Tensor k_new, Tensor v_new, Tensor k, Tensor v,
                                                              Tensor ck, const int32_t *__restrict__ seqlens,
                                                              int32_t n_copy) {
    const int b = blockIdx.z, h = blockIdx.y;
    const int32_t L = seqlens[b];
    if (L < dm.n_q || L > dm.max_seqlen) return;          // a sequence shorter than n_q is skipped as a whole
    const int c = (threadIdx.x & 15) * 8, sub = threadIdx.x >> 4;
    const int32_t first_new = L - dm.n_q;
    if ((int)blockIdx.x < n_copy) {
        const int qi = blockIdx.x * 16 + sub;
        if (qi >= dm.n_q) return;
        const int64_t dst = first_new + qi;
        *reinterpret_cast<uint4 *>(k.ptr + b * k.sb + h * k.sh + dst * k.st + c) =
            *reinterpret_cast<const uint4 *>(k_new.ptr + b * k_new.sb + h * k_new.sh + qi * k_new.st + c);
        *reinterpret_cast<uint4 *>(v.ptr + b * v.sb + h * v.sh + dst * v.st + c) =
            *reinterpret_cast<const uint4 *>(v_new.ptr + b * v_new.sb + h * v_new.sh + qi * v_new.st + c);
        return;
    }
    const int32_t jh = num_kernels(first_new) + ((int)blockIdx.x - n_copy) * 16 + sub;
    if (jh >= num_kernels(L)) return;
    const __bf16 *kb = k.ptr + b * k.sb + h * k.sh + c;
    const __bf16 *nb = k_new.ptr + b * k_new.sb + h * k_new.sh + c;
    bf16x8 x[kKernel];
#pragma unroll
    for (int t = 0; t < kKernel; ++t) {
        const int32_t r = jh * kStride + t;
        x[t] = r >= first_new ? load8(nb + (int64_t)(r - first_new) * k_new.st) : load8(kb + (int64_t)r * k.st);
    }
    double acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0;
#pragma unroll
    for (int t = 0; t < kKernel; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += (double)(float)x[t][e];
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        w[e] = (uint32_t)f64_to_bf16_rne(acc[2 * e] / (double)kKernel) |
               ((uint32_t)f64_to_bf16_rne(acc[2 * e + 1] / (double)kKernel) << 16);
    *reinterpret_cast<uint4 *>(ck.ptr + b * ck.sb + h * ck.sh + (int64_t)jh * ck.st + c) = uint4{w[0], w[1], w[2], w[3]};
}

int launch_append_kv(const Dims &dm, Tensor k_new, Tensor v_new, Tensor k, Tensor v, const Tensor *ck,
                     const int32_t *seqlens, hipStream_t stream) {
    if (ck && dm.n_q > 1) {
        if (dm.batch <= 0) return 0;
        const int n_copy = (dm.n_q + 15) / 16, n_comp = (dm.n_q / kStride + 1 + 15) / 16;
        timing_begin("append_compress_kernel", stream);
        hipLaunchKernelGGL(append_compress_kernel, dim3(n_copy + n_comp, dm.Hkv, dm.batch), dim3(256), 0, stream, dm,
                           k_new, v_new, k, v, *ck, seqlens, n_copy);
        timing_end(stream);
        return (int)hipGetLastError();
    }
    int rows = dm.batch * dm.Hkv * dm.n_q;
    if (rows <= 0) return 0;
    timing_begin("append_kv_kernel", stream);
    if (ck && dm.n_q == 1)
        hipLaunchKernelGGL(append_kv_kernel<true>, dim3((rows + 15) / 16), dim3(256), 0, stream, dm, k_new,
                           v_new, k, v, *ck, seqlens);
    else
        hipLaunchKernelGGL(append_kv_kernel<false>, dim3((rows + 15) / 16), dim3(256), 0, stream, dm, k_new,
                           v_new, k, v, k, seqlens);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
