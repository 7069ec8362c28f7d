// Stage 3, prefill: exact softmax attention of every query token over its own selected
// key-value blocks (section 2.1.1, second stage; section 2.1.3 "Different Granularity for
// Query and Key-Value Tokens": the query unit is a token, the key-value unit a 64-token block).
//
// A workgroup owns 16 consecutive query tokens of one key-value head; each of its 4 wavefronts
// owns 4 of them.  The G (<=16) query heads of a token fill the 16 columns of one MFMA tile, so
// per-token block sets cost no padded matrix work when G = 16.  The workgroup walks the UNION of
// its tokens' block lists in ascending order; each union block is staged in LDS once (K row-major,
// V transposed) and every wavefront runs the two contractions only for those of its tokens that
// selected the block, reusing each LDS fragment it reads across them.
//
// Both contractions are computed transposed so that no register shuffles are needed:
//   S^T[key, head] = K[key, :] . Q[head, :]            A = K tile,   B = Q (held in registers)
//   O^T[c,  head] += V^T[c, key] . P^T[key, head]       A = V^T tile, B = P^T straight from the
// accumulator layout of S^T (lane = head column, 4 consecutive keys per 16-lane group), with the
// key order inside V^T's rows permuted to match.
#include "common.h"

namespace infllmv2 {

constexpr int kQT = 16;        // query tokens per workgroup
constexpr int kTokPerWave = 4;
constexpr int kKPitch = 136;   // bf16 elements per K row in LDS (272 B: conflict-free 16-B reads)
constexpr int kVPitch = 72;    // bf16 elements per V^T row in LDS (144 B)

// Consecutive virtual ids land on the same XCD (hardware deals workgroups round-robin over 8
// XCDs), so neighbouring query tiles -- which share blocks -- share an L2.
__device__ inline uint32_t xcd_contiguous_id(uint32_t bid, uint32_t n) {
    const uint32_t per = n >> 3, rem = n & 7u, x = bid & 7u, slot = bid >> 3;
    return x * per + (x < rem ? x : rem) + slot;
}

__device__ inline int wave_min_i32(int v) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int w = __shfl_xor(v, o);
        v = w < v ? w : v;
    }
    return v;
}

__global__ __launch_bounds__(256) void attn_prefill_kernel(Dims dm, Tensor q, Tensor k, Tensor v,
                                                            const int32_t *__restrict__ seqlens,
                                                            const int32_t *__restrict__ block_idx,
                                                            Tensor out, float *__restrict__ lse,
                                                            int32_t n_tiles) {
    __shared__ __align__(16) __bf16 Ks[kBlock * kKPitch];
    __shared__ __align__(16) __bf16 Vt[kHeadDim * kVPitch];
    __shared__ int next_blk[2][4];

    const uint32_t vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int tile = vid % n_tiles;
    const int h = (vid / n_tiles) % dm.Hkv;
    const int b = vid / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int t0 = tile * kQT;
    if (t0 >= L) return;                       // whole tile beyond the sequence (uniform)
    const int b_own = t0 / kBlock;             // the tile's own block: the only one with a causal edge

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;    // MFMA column (query head) and 16-lane group
    const int G = dm.G;

    // ---- per-wave state: 4 tokens ------------------------------------------------------------
    bf16x8 qf[kTokPerWave][4];
    f32x4 o[kTokPerWave][8];
    float m_run[kTokPerWave], l_run[kTokPerWave];
    int own[kTokPerWave];                      // lane e < topk holds entry e of the token's block list
#pragma unroll
    for (int u = 0; u < kTokPerWave; ++u) {
        const int tok = t0 + wave * kTokPerWave + u;
        const bool live = tok < L;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[u][ks] = zero8();
            if (live && n < G)
                qf[u][ks] = load8(q.ptr + b * q.sb + (int64_t)tok * q.st + (int64_t)(h * G + n) * q.sh +
                                  32 * ks + 8 * g);
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[u][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run[u] = -INFINITY;
        l_run[u] = 0.f;
        int e = 0x7fffffff;
        if (live && lane < dm.topk) {
            int x = block_idx[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * dm.topk + lane];
            if (x >= 0 && x <= b_own) e = x;
        }
        own[u] = e;
    }

    const __bf16 *kbase = k.ptr + b * k.sb + h * k.sh;
    const __bf16 *vbase = v.ptr + b * v.sb + h * v.sh;
    const int sc = tid & 15;                   // staging: 16-byte chunk within a 256-byte row
    const int sr = tid >> 4;                   // staging: row group

    int cur = -1;
    for (int it = 0;; ++it) {
        // ---- next block of the union: smallest entry above the current one --------------------
        int cand = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < kTokPerWave; ++u) {
            int e = own[u] > cur ? own[u] : 0x7fffffff;
            cand = e < cand ? e : cand;
        }
        cand = wave_min_i32(cand);
        if (lane == 0) next_blk[it & 1][wave] = cand;
        __syncthreads();                       // also: everyone is done with the previous tiles
        int blk = next_blk[it & 1][0];
#pragma unroll
        for (int w = 1; w < 4; ++w) blk = next_blk[it & 1][w] < blk ? next_blk[it & 1][w] : blk;
        if (blk == 0x7fffffff) break;
        cur = blk;

        // ---- stage K (row-major) and V (transposed, key-permuted) of this block -----------------
        const int key0 = blk * kBlock;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = sr + 16 * i;
            uint4 x = {0u, 0u, 0u, 0u};
            if (key0 + r < L) x = *reinterpret_cast<const uint4 *>(kbase + (int64_t)(key0 + r) * k.st + 8 * sc);
            *reinterpret_cast<uint4 *>(&Ks[r * kKPitch + 8 * sc]) = x;
        }
        {
            // thread = 4 consecutive keys (4*sr ..) x 8 channels (8*sc ..)
            uint4 x[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = uint4{0u, 0u, 0u, 0u};
                const int r = 4 * sr + i;
                if (key0 + r < L) x[i] = *reinterpret_cast<const uint4 *>(vbase + (int64_t)(key0 + r) * v.st + 8 * sc);
            }
            // keys 4*sr..4*sr+3 sit at slots 32*(sr/8) + 8*(sr%4) + 4*((sr%8)/4) .. +3 of a V^T row
            const int slot = 32 * (sr >> 3) + 8 * (sr & 3) + 4 * ((sr & 7) >> 2);
            const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&x[0]);
            const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&x[1]);
            const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&x[2]);
            const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&x[3]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {      // channel pair (2e, 2e+1)
                uint2 lo, hi;                  // lo: channel 2e of keys 0..3, hi: channel 2e+1
                lo.x = (w0[e] & 0xffffu) | (w1[e] << 16);
                lo.y = (w2[e] & 0xffffu) | (w3[e] << 16);
                hi.x = (w0[e] >> 16) | (w1[e] & 0xffff0000u);
                hi.y = (w2[e] >> 16) | (w3[e] & 0xffff0000u);
                *reinterpret_cast<uint2 *>(&Vt[(8 * sc + 2 * e) * kVPitch + slot]) = lo;
                *reinterpret_cast<uint2 *>(&Vt[(8 * sc + 2 * e + 1) * kVPitch + slot]) = hi;
            }
        }
        __syncthreads();

        // ---- which of this wave's tokens selected the block -----------------------------------
        bool member[kTokPerWave];
        bool any_member = false;
#pragma unroll
        for (int u = 0; u < kTokPerWave; ++u) {
            member[u] = __ballot(own[u] == blk) != 0ull;
            any_member |= member[u];
        }
        if (!any_member) continue;

        // ---- S^T = K . Q^T for the member tokens, K fragments read once --------------------------
        f32x4 s[kTokPerWave][4];
#pragma unroll
        for (int u = 0; u < kTokPerWave; ++u)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) s[u][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                bf16x8 a = load8(&Ks[(16 * mt + n) * kKPitch + 32 * ks + 8 * g]);
#pragma unroll
                for (int u = 0; u < kTokPerWave; ++u)
                    if (member[u]) s[u][mt] = mfma16(a, qf[u][ks], s[u][mt]);
            }

        // ---- online softmax per (token, head); P^T packed to bf16 in MFMA B layout --------------
        bf16x8 pf[kTokPerWave][2];
        const bool edge = (blk == b_own) || (key0 + kBlock > L);
#pragma unroll
        for (int u = 0; u < kTokPerWave; ++u) {
            if (!member[u]) continue;
            const int tok = t0 + wave * kTokPerWave + u;
            float mx = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float x = s[u][mt][j] * dm.scale_log2;
                    if (edge && key0 + 16 * mt + 4 * g + j > tok) x = -INFINITY;
                    s[u][mt][j] = x;
                    mx = fmaxf(mx, x);
                }
            mx = xgroup_max(mx);
            const float m_new = fmaxf(m_run[u], mx);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = fast_exp2(m_run[u] - m_use);
            float psum = 0.f;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float p = fast_exp2(s[u][mt][j] - m_use);
                    s[u][mt][j] = p;
                    psum += p;
                }
            l_run[u] = l_run[u] * alpha + psum;
            m_run[u] = m_new;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[u][dt] *= alpha;
            }
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                bf16x8 p8;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    p8[j] = (__bf16)s[u][2 * kk][j];
                    p8[4 + j] = (__bf16)s[u][2 * kk + 1][j];
                }
                pf[u][kk] = p8;
            }
        }

        // ---- O^T += V^T . P^T, V fragments read once -------------------------------------------
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                bf16x8 a = load8(&Vt[(16 * dt + n) * kVPitch + 32 * kk + 8 * g]);
#pragma unroll
                for (int u = 0; u < kTokPerWave; ++u)
                    if (member[u]) o[u][dt] = mfma16(a, pf[u][kk], o[u][dt]);
            }
    }

    // ---- normalise and write: lane holds channels 16*dt + 4*g .. +3 of head n ------------------
#pragma unroll
    for (int u = 0; u < kTokPerWave; ++u) {
        const int tok = t0 + wave * kTokPerWave + u;
        if (tok >= L || n >= G) continue;
        const float l_tot = xgroup_sum(l_run[u]);
        const float inv = 1.f / l_tot;
        __bf16 *op = out.ptr + b * out.sb + (int64_t)tok * out.st + (int64_t)(h * G + n) * out.sh + 4 * g;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            bf16x4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = (__bf16)(o[u][dt][j] * inv);
            *reinterpret_cast<uint2 *>(op + 16 * dt) = __builtin_bit_cast(uint2, r);
        }
        if (g == 0)
            lse[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + n] = (m_run[u] + fast_log2(l_tot)) * kLn2;
    }
}

int launch_attn_prefill(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                        const int32_t *block_idx, Tensor out, float *lse, hipStream_t stream) {
    const int32_t n_tiles = (dm.max_seqlen + kQT - 1) / kQT;
    const int64_t n_wg = (int64_t)n_tiles * dm.Hkv * dm.batch;
    if (n_wg <= 0) return 0;
    timing_begin("attn_prefill_kernel", stream);
    hipLaunchKernelGGL(attn_prefill_kernel, dim3((uint32_t)n_wg), dim3(256), 0, stream, dm, q, k, v,
                       seqlens, block_idx, out, lse, n_tiles);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
