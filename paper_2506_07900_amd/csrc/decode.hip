// Decode step, stages 2 and 3 for ONE query token per sequence at position seqlens[b]-1
// (section 2.1.3 "Different Granularity for Query and Key-Value Tokens": token-level queries
// keep the method usable in decoding; section 5.4: per step the attended blocks stay constant
// and only the semantic-kernel representations grow).
//
// Selection: G x n_c logits per key-value head.  The softmax needs the log-sum-exp over ALL
// visible kernels before any score can be ranked, so the scan is split:
//   decode_logits_kernel   every CU takes 64 kernels: MFMA logits -> scratch, per-16-kernel
//                          partial (max, sum) per head
//   decode_topk_kernel     one workgroup per (sequence, key-value head): merges the partials
//                          into the log-sum-exp, forms group-mean scores, 5/4 max-pool to
//                          blocks, forces initial/local blocks, ordered top-k
// Attention: one workgroup per selected block (split-KV) writes an unnormalised partial
// (o, max, sum); decode_merge_kernel combines the k partials per query head.
#include "common.h"

namespace infllmv2 {

__device__ inline int clamp_len(int32_t L, int32_t cap) { return L < 0 ? 0 : (L > cap ? cap : L); }

// ---- selection, part 1 ------------------------------------------------------------------------
// grid (ceil(n_c_cap/64), Hkv, B); wave w of a workgroup owns kernels 64*bx + 16*w .. +15.
// Z^T = CK . Q^T: lane = query head, 4 accumulator entries = 4 consecutive kernels.
__global__ __launch_bounds__(256) void decode_logits_kernel(Dims dm, Tensor q, Tensor ck,
                                                             const int32_t *__restrict__ seqlens,
                                                             float *__restrict__ zbuf,
                                                             float2 *__restrict__ part, int32_t n_c_cap,
                                                             int32_t n_part) {
    const int b = blockIdx.z, h = blockIdx.y;
    const int L = clamp_len(seqlens[b], dm.max_seqlen);
    const int n_vis = num_kernels(L);                 // the query sits at L-1: n_c((L-1)+1)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int jh0 = blockIdx.x * 64 + wave * 16;
    if (jh0 >= n_vis) return;
    const int G = dm.G;
    f32x4 z = {0.f, 0.f, 0.f, 0.f};
    const __bf16 *ckr = ck.ptr + b * ck.sb + h * ck.sh + (int64_t)(jh0 + n) * ck.st + 8 * g;
    const __bf16 *qr = q.ptr + b * q.sb + (int64_t)(h * G + n) * q.sh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8 a = zero8(), bq = zero8();
        if (jh0 + n < n_vis) a = load8(ckr + 32 * ks);
        if (n < G) bq = load8(qr + 32 * ks);
        z = mfma16(a, bq, z);
    }
    float mx = -INFINITY;
    float x[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[j] = z[j] * dm.scale_log2;
        if (jh0 + 4 * g + j >= n_vis) x[j] = -INFINITY;
        mx = fmaxf(mx, x[j]);
    }
    mx = xgroup_max(mx);                              // finite: kernel jh0 is visible
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) s += fast_exp2(x[j] - mx);
    s = xgroup_sum(s);
    if (n < G) {
        float *zr = zbuf + (((int64_t)b * dm.Hkv + h) * G + n) * n_c_cap + jh0 + 4 * g;
        *reinterpret_cast<float4 *>(zr) = float4{x[0], x[1], x[2], x[3]};
        if (g == 0) part[(((int64_t)b * dm.Hkv + h) * G + n) * n_part + (jh0 >> 4)] = float2{mx, s};
    }
}

// Ordered argmax over a workgroup: (score descending, index ascending).
__device__ inline void wave_best(float &s, int &j) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float os = __shfl_xor(s, o);
        const int oj = __shfl_xor(j, o);
        if (os > s || (os == s && oj < j)) {
            s = os;
            j = oj;
        }
    }
}

// ---- selection, part 2 ------------------------------------------------------------------------
// grid (Hkv, B), 1024 threads.  Dynamic LDS: r[n_c_cap + 1] kernel scores (slot 0 = kernel -1),
// R[nb_cap] block scores.
__global__ __launch_bounds__(1024) void decode_topk_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                            const float *__restrict__ zbuf,
                                                            const float2 *__restrict__ part,
                                                            int32_t n_c_cap, int32_t n_part, int32_t nb_cap,
                                                            int32_t *__restrict__ block_idx) {
    extern __shared__ float smem[];
    float *r = smem;                        // [n_c_cap + 1]
    float *R = smem + n_c_cap + 1;          // [nb_cap]
    __shared__ float lse_h[16];
    __shared__ float best_s[16];
    __shared__ int best_j[16];
    __shared__ int picks[kMaxTopk];
    const int h = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = dm.G;
    const int L = clamp_len(seqlens[b], dm.max_seqlen);
    int32_t *out = block_idx + ((int64_t)b * dm.Hkv + h) * dm.topk;
    if (L < 1) {
        if (tid < dm.topk) out[tid] = -1;
        return;
    }
    const int n_vis = num_kernels(L);
    const int np = (n_vis + 15) >> 4;       // valid partials
    const int b_own = (L - 1) / kBlock, n_blk = b_own + 1;

    // log-sum-exp per head: wave w reduces head w (16 waves, up to 16 heads)
    if (wave < G) {
        const float2 *pp = part + (((int64_t)b * dm.Hkv + h) * G + wave) * n_part;
        float m = -INFINITY;
        for (int i = lane; i < np; i += 64) m = fmaxf(m, pp[i].x);
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
        float s = 0.f;
        for (int i = lane; i < np; i += 64) {
            float2 v = pp[i];
            s += v.y * fast_exp2(v.x - m);
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) s += __shfl_xor(s, o);
        if (lane == 0) lse_h[wave] = np > 0 ? m + fast_log2(s) : 0.f;
    }
    __syncthreads();
    // group-mean kernel scores
    const float *zb = zbuf + ((int64_t)b * dm.Hkv + h) * G * n_c_cap;
    const float inv_g = 1.f / G;
    for (int jh = tid; jh < n_vis; jh += 1024) {
        float acc = 0.f;
        for (int gq = 0; gq < G; ++gq) acc += fast_exp2(zb[(int64_t)gq * n_c_cap + jh] - lse_h[gq]);
        r[jh + 1] = fmaxf(acc * inv_g, kScoreFloor);
    }
    if (tid == 0) r[0] = -INFINITY;
    __syncthreads();
    // block scores: kernels 4j-1 .. 4j+3 that are visible; forced blocks to +inf
    for (int j = tid; j < n_blk; j += 1024) {
        float v = -INFINITY;
#pragma unroll
        for (int x = 0; x < 5; ++x) {
            const int jh = 4 * j - 1 + x;
            if (jh < n_vis) v = fmaxf(v, r[jh + 1]);
        }
        if (j < dm.n_init || j > b_own - dm.n_local) v = INFINITY;
        R[j] = v;
    }
    __syncthreads();
    const int n_sel = dm.topk < n_blk ? dm.topk : n_blk;
    float last_s = INFINITY;
    int last_j = -1;
    for (int c = 0; c < n_sel; ++c) {
        float bs = -INFINITY;
        int bj = 0x7fffffff;
        for (int j = tid; j < n_blk; j += 1024) {
            const float sc = R[j];
            const bool after = sc < last_s || (sc == last_s && j > last_j);
            if (after && (sc > bs || (sc == bs && j < bj))) {
                bs = sc;
                bj = j;
            }
        }
        wave_best(bs, bj);
        if (lane == 0) {
            best_s[wave] = bs;
            best_j[wave] = bj;
        }
        __syncthreads();
        bs = best_s[0];
        bj = best_j[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) {
            const float os = best_s[w];
            const int oj = best_j[w];
            if (os > bs || (os == bs && oj < bj)) {
                bs = os;
                bj = oj;
            }
        }
        last_s = bs;
        last_j = bj;
        if (tid == 0) picks[c] = bj;
        __syncthreads();
    }
    if (tid < dm.topk) {
        if (tid < n_sel) {
            const int mine = picks[tid];
            int rank = 0;
            for (int c = 0; c < n_sel; ++c) rank += picks[c] < mine ? 1 : 0;
            out[rank] = mine;
        } else {
            out[tid] = -1;
        }
    }
}

// ---- attention, part 1: one workgroup per selected block --------------------------------------
// grid (topk, Hkv, B).  Wave w: keys 16w..16w+15 of the block, S^T = K . Q^T on MFMA; then
// thread (head, 8-channel chunk) accumulates p*v over the 64 keys in fp32.
__global__ __launch_bounds__(256) void decode_attn_partial_kernel(Dims dm, Tensor q, Tensor k, Tensor v,
                                                                   const int32_t *__restrict__ seqlens,
                                                                   const int32_t *__restrict__ block_idx,
                                                                   float *__restrict__ o_part,
                                                                   float2 *__restrict__ ml_part) {
    __shared__ float S[kBlock][17];
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int G = dm.G;
    const int L = clamp_len(seqlens[b], dm.max_seqlen);
    const int blk = block_idx[((int64_t)b * dm.Hkv + h) * dm.topk + c];
    const int head = tid & 15, chunk = tid >> 4;
    const int64_t pbase = (((int64_t)b * dm.Hq + h * G + head) * dm.topk + c);
    const bool valid = L >= 1 && blk >= 0 && (int64_t)blk * kBlock < L;
    if (!valid) {                                        // uniform over the workgroup
        if (head < G) {
            if (chunk == 0) ml_part[pbase] = float2{-INFINITY, 0.f};
            float4 zf = {0.f, 0.f, 0.f, 0.f};
            float4 *op = reinterpret_cast<float4 *>(o_part + pbase * kHeadDim + 8 * chunk);
            op[0] = zf;
            op[1] = zf;
        }
        return;
    }
    const int key0 = blk * kBlock;
    const int pos = L - 1;
    {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        const int key = key0 + 16 * wave + n;
        const __bf16 *kr = k.ptr + b * k.sb + h * k.sh + (int64_t)key * k.st + 8 * g;
        const __bf16 *qr = q.ptr + b * q.sb + (int64_t)(h * G + n) * q.sh + 8 * g;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 a = zero8(), bq = zero8();
            if (key <= pos) a = load8(kr + 32 * ks);
            if (n < G) bq = load8(qr + 32 * ks);
            s = mfma16(a, bq, s);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int kk = 16 * wave + 4 * g + j;
            S[kk][n] = (key0 + kk <= pos) ? s[j] * dm.scale_log2 : -INFINITY;
        }
    }
    __syncthreads();
    if (head >= G) return;
    float m = -INFINITY;
#pragma unroll 8
    for (int kk = 0; kk < kBlock; ++kk) m = fmaxf(m, S[kk][head]);     // key0 <= pos: finite
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    float l = 0.f;
    const int n_keys = min(kBlock, pos - key0 + 1);
    const __bf16 *vr = v.ptr + b * v.sb + h * v.sh + (int64_t)key0 * v.st + 8 * chunk;
#pragma unroll 4
    for (int kk = 0; kk < n_keys; ++kk) {
        const float p = fast_exp2(S[kk][head] - m);
        l += p;
        bf16x8 x = load8(vr + (int64_t)kk * v.st);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += p * (float)x[e];
    }
    if (chunk == 0) ml_part[pbase] = float2{m, l};
    float4 *op = reinterpret_cast<float4 *>(o_part + pbase * kHeadDim + 8 * chunk);
    op[0] = float4{acc[0], acc[1], acc[2], acc[3]};
    op[1] = float4{acc[4], acc[5], acc[6], acc[7]};
}

// ---- attention, part 2: merge the k partials of every query head ---------------------------------
// grid (Hq, B), 128 threads: thread = channel.
__global__ __launch_bounds__(128) void decode_merge_kernel(Dims dm, const float *__restrict__ o_part,
                                                            const float2 *__restrict__ ml_part, Tensor out,
                                                            float *__restrict__ lse) {
    const int hq = blockIdx.x, b = blockIdx.y, cch = threadIdx.x;
    const int64_t pbase = ((int64_t)b * dm.Hq + hq) * dm.topk;
    float M = -INFINITY;
    for (int c = 0; c < dm.topk; ++c) M = fmaxf(M, ml_part[pbase + c].x);
    float num = 0.f, den = 0.f;
    if (M > -INFINITY) {
        for (int c = 0; c < dm.topk; ++c) {
            const float2 ml = ml_part[pbase + c];
            const float w = fast_exp2(ml.x - M);
            den += w * ml.y;
            num += w * o_part[(pbase + c) * kHeadDim + cch];
        }
    }
    const float o = den > 0.f ? num / den : 0.f;
    out.ptr[b * out.sb + (int64_t)hq * out.sh + cch] = (__bf16)o;
    if (cch == 0) lse[(int64_t)b * dm.Hq + hq] = den > 0.f ? (M + fast_log2(den)) * kLn2 : -INFINITY;
}

// ---- host side -------------------------------------------------------------------------------------
static inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

struct DecodeSelLayout {
    int32_t n_c_cap, n_part, nb_cap;
    size_t z_bytes, part_bytes;
};
static DecodeSelLayout decode_sel_layout(const Dims &dm) {
    DecodeSelLayout l;
    int32_t n_c = num_kernels(dm.max_seqlen);
    l.n_c_cap = (n_c + 63) / 64 * 64;
    if (l.n_c_cap < 64) l.n_c_cap = 64;
    l.n_part = l.n_c_cap / 16;
    l.nb_cap = (dm.max_seqlen + kBlock - 1) / kBlock + 1;
    l.z_bytes = align256((size_t)dm.batch * dm.Hq * l.n_c_cap * sizeof(float));
    l.part_bytes = align256((size_t)dm.batch * dm.Hq * l.n_part * sizeof(float2));
    return l;
}

size_t select_decode_ws_bytes(const Dims &dm) {
    DecodeSelLayout l = decode_sel_layout(dm);
    return l.z_bytes + l.part_bytes;
}

size_t select_decode_lds_bytes(const Dims &dm) {
    DecodeSelLayout l = decode_sel_layout(dm);
    return ((size_t)l.n_c_cap + 1 + l.nb_cap) * sizeof(float);
}

int launch_select_decode(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                         int32_t *block_idx, void *ws, hipStream_t stream) {
    if (dm.batch <= 0) return 0;
    DecodeSelLayout l = decode_sel_layout(dm);
    float *zbuf = reinterpret_cast<float *>(ws);
    float2 *part = reinterpret_cast<float2 *>(reinterpret_cast<char *>(ws) + l.z_bytes);
    timing_begin("decode_logits_kernel", stream);
    hipLaunchKernelGGL(decode_logits_kernel, dim3(l.n_c_cap / 64, dm.Hkv, dm.batch), dim3(256), 0,
                       stream, dm, q, ck, seqlens, zbuf, part, l.n_c_cap, l.n_part);
    timing_end(stream);
    const size_t lds = select_decode_lds_bytes(dm);
    timing_begin("decode_topk_kernel", stream);
    hipLaunchKernelGGL(decode_topk_kernel, dim3(dm.Hkv, dm.batch), dim3(1024), lds, stream, dm, seqlens,
                       zbuf, part, l.n_c_cap, l.n_part, l.nb_cap, block_idx);
    timing_end(stream);
    return (int)hipGetLastError();
}

size_t attn_decode_ws_bytes(const Dims &dm) {
    const size_t o = align256((size_t)dm.batch * dm.Hq * dm.topk * kHeadDim * sizeof(float));
    const size_t ml = align256((size_t)dm.batch * dm.Hq * dm.topk * sizeof(float2));
    return o + ml;
}

int launch_attn_decode(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                       const int32_t *block_idx, Tensor out, float *lse, void *ws, hipStream_t stream) {
    if (dm.batch <= 0) return 0;
    const size_t o_bytes = align256((size_t)dm.batch * dm.Hq * dm.topk * kHeadDim * sizeof(float));
    float *o_part = reinterpret_cast<float *>(ws);
    float2 *ml_part = reinterpret_cast<float2 *>(reinterpret_cast<char *>(ws) + o_bytes);
    timing_begin("decode_attn_partial_kernel", stream);
    hipLaunchKernelGGL(decode_attn_partial_kernel, dim3(dm.topk, dm.Hkv, dm.batch), dim3(256), 0, stream,
                       dm, q, k, v, seqlens, block_idx, o_part, ml_part);
    timing_end(stream);
    timing_begin("decode_merge_kernel", stream);
    hipLaunchKernelGGL(decode_merge_kernel, dim3(dm.Hq, dm.batch), dim3(128), 0, stream, dm, o_part,
                       ml_part, out, lse);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
