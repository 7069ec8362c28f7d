// Decode step, stages 2 and 3 for ONE query token per sequence at position seqlens[b]-1
// (section 2.1.3 "Different Granularity for Query and Key-Value Tokens": token-level queries
// keep the method usable in decoding; section 5.4: per step the attended blocks stay constant
// and only the semantic-kernel representations grow), and for the n drafted tokens of a
// speculative-verification step (section 4.1, "InfLLM v2 for Target Model"): the same kernels
// over n query rows per sequence, with the causal test of the last n x n region replaced by a
// bit-packed tree mask.
//
// A decode step moves a few megabytes, so it is bound by launch and memory latency, not by
// bandwidth: every kernel below spreads its reads over many workgroups and issues all the loads
// of a thread before using any of them.
//
// Selection (the softmax needs the log-sum-exp over ALL visible kernels before any score exists):
//   decode_logits_kernel   64 kernels per workgroup: MFMA logits, one partial (max, sum) per head
//                          and workgroup
//   decode_scores_*kernel  merges the partials into the log-sum-exp, group-mean scores, 5/4 max-pool
//                          -> block scores; the logits come from scratch (plain decode) or are
//                          computed again on the matrix cores (verification)
//   decode_pick_kernel     two-level top-k of the block-score row
// Attention: one workgroup per selected block (split-KV) writes an unnormalised partial
// (o, max, sum); decode_merge_kernel combines the k partials per query head.  The one-call steps
// run the top-k inside the attention kernel (decode_pick_partial_kernel): one launch fewer.
#include "common.h"

namespace infllmv2 {

__device__ inline int clamp_len(int32_t L, int32_t cap) { return L < 0 ? 0 : (L > cap ? cap : L); }

// Every kernel below works on "query rows": row bv = b * n_q + qi is query token qi of sequence b.
// Plain decode has n_q = 1.  Draft verification (section 4.1, "InfLLM v2 for Target Model") has the
// n_q drafted tokens in the last n_q cache rows; token qi sits at position seqlens[b] - n_q + qi and
// selects blocks like any query at that position.  Returns the number of cache rows up to and
// including the query (0: the row is skipped; a sequence shorter than n_q is skipped as a whole).
__device__ inline int query_row(const Dims &dm, const int32_t *__restrict__ seqlens, int bv, int &b, int &qi) {
    if (dm.n_q == 1) {
        b = bv;
        qi = 0;
        return clamp_len(seqlens[b], dm.max_seqlen);
    }
    b = bv / dm.n_q;
    qi = bv - b * dm.n_q;
    const int L_all = clamp_len(seqlens[b], dm.max_seqlen);
    return L_all < dm.n_q ? 0 : L_all - (dm.n_q - 1 - qi);
}

// Query operands of parts 1 and 2.  MFMA operand layout: lane (n, g) holds head n, channels
// 32*ks + 8*g .. +7.  One query per workgroup: straight from memory.  Several (verification): every
// wave needs the same rows and every workgroup of the launch the same few cache lines, so the
// workgroup fetches them once into LDS (row pitch 272 bytes: conflict-free 16-byte reads).
constexpr int kQsPitch = kHeadDim + 8;
template <int kQT>
__device__ inline void load_query_operands(const Dims &dm, const Tensor &q, int b, int h, int qi0, uint16_t *qs,
                                           bf16x8 (&bq)[kQT][4]) {
    const int lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;
    const int G = dm.G;
    if constexpr (kQT == 1) {
        const __bf16 *qr = q.ptr + b * q.sb + min(qi0, dm.n_q - 1) * q.st + (int64_t)(h * G + min(n, G - 1)) * q.sh + 8 * g;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) bq[0][ks] = load8(qr + 32 * ks);
    } else {
        const int row = threadIdx.x >> 4, c16 = threadIdx.x & 15;     // 256 threads: 16 heads x 16 chunks of 16 bytes
        uint4 x[kQT];
#pragma unroll
        for (int t = 0; t < kQT; ++t)
            x[t] = *reinterpret_cast<const uint4 *>(q.ptr + b * q.sb + min(qi0 + t, dm.n_q - 1) * q.st +
                                                    (int64_t)(h * G + min(row, G - 1)) * q.sh + 8 * c16);
#pragma unroll
        for (int t = 0; t < kQT; ++t) *reinterpret_cast<uint4 *>(&qs[(t * 16 + row) * kQsPitch + 8 * c16]) = x[t];
        __syncthreads();
#pragma unroll
        for (int t = 0; t < kQT; ++t)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                bq[t][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&qs[(t * 16 + n) * kQsPitch + 32 * ks + 8 * g]));
    }
}

// ---- selection, parts 1 and 2 -------------------------------------------------------------------
// Both parts score semantic kernels against kQT consecutive query tokens of one sequence on the
// matrix cores.  kQT = 1 is plain decode; verification uses kQT = kVerifyQT.  A workgroup of part 1
// covers kTW tiles of 16 kernels per wave, one of part 2 tiles_per_wave2 (plus one halo tile).  More
// tiles per wave mean fewer workgroups and fewer log-sum-exp partials for part 2 to merge (every
// workgroup of part 2 reads all partials of its heads); fewer tiles spread a lone step over more compute
// units.  Measured at 128K context, plain decode, 1 / 2 / 4 tiles: 21.6 / 21.1 / 21.6 us per step for
// one sequence, 27.2 / 26.8 / 25.8 us for the ragged batch of 8, 73 / 62 / 61 us for 32 sequences (eight
// tiles: 63 us);
// verification (4 to 64 drafted tokens): under 10 % between them.
constexpr int kVerifyQT = 4;
__host__ __device__ constexpr int tiles_per_wave(int qt) { return 2; }                   // part 1, verification
// part 1, plain decode: by batch size
static inline int decode_tiles_per_wave(const Dims &dm) { return dm.batch >= 4 ? 4 : 2; }
__host__ __device__ constexpr int tiles_per_wave2(int qt) { return qt == 1 ? 1 : 2; }   // part 2

// length of the cache up to and including query token qi of sequence b (0: no such row)
__device__ inline int row_len(const Dims &dm, int L_all, int qi) {
    return (L_all < dm.n_q || qi >= dm.n_q) ? 0 : L_all - (dm.n_q - 1 - qi);
}

// Channels c0 .. c0+7 of the semantic kernel that the token appended at position L-1 completes: rows
// L-32 .. L-2 from the cache, row L-1 from the step's new key; fp64 sum in token order, one rounding
// (the bits compress_keys_kernel produces once the row is in the cache).
__device__ inline bf16x8 fresh_kernel_row8(const AppendArgs &ap, int b, int h, int L, int c0) {
    const __bf16 *kc = ap.k.ptr + b * ap.k.sb + h * ap.k.sh + c0;
    double acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0;
#pragma unroll 1
    for (int t0 = 0; t0 < kKernel; t0 += 8) {            // eight rows in flight at a time
        bf16x8 rows[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            rows[i] = t0 + i < kKernel - 1 ? load8(kc + (int64_t)(L - kKernel + t0 + i) * ap.k.st)
                                           : load8(ap.k_new.ptr + b * ap.k_new.sb + h * ap.k_new.sh + c0);
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (double)(float)rows[i][e];
    }
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        w[e] = (uint32_t)f64_to_bf16_rne(acc[2 * e] / (double)kKernel) |
               ((uint32_t)f64_to_bf16_rne(acc[2 * e + 1] / (double)kKernel) << 16);
    return __builtin_bit_cast(bf16x8, uint4{w[0], w[1], w[2], w[3]});
}

// ---- part 1: partial (max, sum) of the relevance softmax ---------------------------------------------
// grid (n_c_cap / (64*kTW), Hkv, B * ceil(n_q/kQT)); wave w owns kernels chunk + 16*kTW*w .. +16*kTW-1.
// Z^T = CK . Q^T: lane = query head, 4 accumulator entries = 4 consecutive kernels.
// With kAppend (plain decode, the fused step) the kernel also opens the step: the workgroups of chunk 0
// copy the new token's key and value rows into the caches (nothing before the attention kernel reads
// them), and the wave that owns the semantic kernel the new token completes builds its representation
// itself -- 31 cached rows and the new one, fp64 sum in token order, one rounding, the same bits as
// compress_keys_kernel -- uses it, and stores it for the steps to come.
template <int kQT, bool kAppend, int kTW>
__global__ __launch_bounds__(256) void decode_logits_kernel(Dims dm, Tensor q, Tensor ck,
                                                             const int32_t *__restrict__ seqlens,
                                                             float *__restrict__ zbuf, int32_t n_c_cap,
                                                             float2 *__restrict__ part,
                                                             float2 *__restrict__ part_c, int32_t n_part,
                                                             AppendArgs ap) {
    static_assert(!kAppend || kQT == 1, "the fused append is for one query per sequence");
    constexpr int kChunk = 64 * kTW;
    __shared__ float2 wpart[kQT][4][16];
    __shared__ float2 wpart_c[kQT][4][16];
    __shared__ __align__(16) uint16_t qs[kQT > 1 ? kQT * 16 * kQsPitch : 8];
    __shared__ __align__(16) uint32_t newrow[kAppend ? 64 : 1];
    const int h = blockIdx.y;
    const int n_qt = (dm.n_q + kQT - 1) / kQT;        // query tiles per sequence
    const int b = kQT == 1 ? blockIdx.z : blockIdx.z / n_qt;   // kQT = 1 is only launched with n_q = 1
    const int qi0 = (blockIdx.z - b * n_qt) * kQT;
    const int L_all = clamp_len(seqlens[b], dm.max_seqlen);
    bool closes = false;                              // the new token completes semantic kernel n_vis - 1
    if constexpr (kAppend) {
        const int32_t L_raw = seqlens[b];
        const bool live = L_raw >= 1 && L_raw <= dm.max_seqlen;       // as the stand-alone append: others are skipped
        if (live && blockIdx.x == 0 && threadIdx.x < 32) {
            const int c8 = (threadIdx.x & 15) * 8;
            const Tensor &src = threadIdx.x < 16 ? ap.k_new : ap.v_new;
            const Tensor &dst = threadIdx.x < 16 ? ap.k : ap.v;
            *reinterpret_cast<uint4 *>(dst.ptr + b * dst.sb + h * dst.sh + (int64_t)(L_raw - 1) * dst.st + c8) =
                *reinterpret_cast<const uint4 *>(src.ptr + b * src.sb + h * src.sh + c8);
        }
        closes = live && L_raw >= kKernel && (L_raw - kKernel) % kStride == 0;
    }
    int n_vis[kQT], n_vis_max = 0;                    // query slot t sits at L-1: n_c((L-1)+1); 0 = no such row
#pragma unroll
    for (int t = 0; t < kQT; ++t) {
        n_vis[t] = num_kernels(row_len(dm, L_all, qi0 + t));
        n_vis_max = max(n_vis_max, n_vis[t]);
    }
    if ((int)blockIdx.x * kChunk >= n_vis_max) return;    // uniform over the workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int jw = blockIdx.x * kChunk + wave * 16 * kTW; // first kernel of this wave
    const int G = dm.G;
    bf16x8 a[kTW][4], bq[kQT][4];
#pragma unroll
    for (int i = 0; i < kTW; ++i) {
        const __bf16 *ckr = ck.ptr + b * ck.sb + h * ck.sh + (int64_t)(jw + 16 * i + n) * ck.st + 8 * g;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            a[i][ks] = zero8();
            if (jw + 16 * i + n < n_vis_max) a[i][ks] = load8(ckr + 32 * ks);
        }
    }
    load_query_operands<kQT>(dm, q, b, h, qi0, qs, bq);   // heads >= G repeat head G-1: their columns are never used
    if constexpr (kAppend) {
        const int jh_new = n_vis_max - 1;             // = (L - p) / s when the new token closes a kernel
        if (closes && jh_new >= jw && jh_new < jw + 16 * kTW) {       // uniform over the wave
            // lane = channels 2*lane, 2*lane+1: rows L-32 .. L-2 from the cache, row L-1 from k_new
            const int L = L_all;
            const __bf16 *kc = ap.k.ptr + b * ap.k.sb + h * ap.k.sh + 2 * lane;
            uint32_t rowv[kKernel];
#pragma unroll
            for (int t = 0; t < kKernel - 1; ++t)
                rowv[t] = *reinterpret_cast<const uint32_t *>(kc + (int64_t)(L - kKernel + t) * ap.k.st);
            rowv[kKernel - 1] = *reinterpret_cast<const uint32_t *>(ap.k_new.ptr + b * ap.k_new.sb + h * ap.k_new.sh + 2 * lane);
            double s0 = 0.0, s1 = 0.0;
#pragma unroll
            for (int t = 0; t < kKernel; ++t) {
                s0 += (double)__uint_as_float(rowv[t] << 16);
                s1 += (double)__uint_as_float(rowv[t] & 0xffff0000u);
            }
            const uint32_t packed = (uint32_t)f64_to_bf16_rne(s0 / (double)kKernel) |
                                    ((uint32_t)f64_to_bf16_rne(s1 / (double)kKernel) << 16);
            newrow[lane] = packed;
            *reinterpret_cast<uint32_t *>(ck.ptr + b * ck.sb + h * ck.sh + (int64_t)jh_new * ck.st + 2 * lane) = packed;
            // same wavefront wrote newrow: LDS keeps the order.  The lanes whose operand row it is take it from there.
#pragma unroll
            for (int i = 0; i < kTW; ++i)
                if (jw + 16 * i + n == jh_new) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        a[i][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&newrow[16 * ks + 4 * g]));
                }
        }
    }
#pragma unroll
    for (int t = 0; t < kQT; ++t) {
        float x[kTW][4], mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < kTW; ++i) {
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) z = mfma16(a[i][ks], bq[t][ks], z);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[i][j] = z[j] * dm.scale_log2;
                if (jw + 16 * i + 4 * g + j >= n_vis[t]) x[i][j] = -INFINITY;
                mx = fmaxf(mx, x[i][j]);
            }
        }
        mx = xgroup_max(mx);
        const float m_use = mx == -INFINITY ? 0.f : mx;
        float sm = 0.f;
#pragma unroll
        for (int i = 0; i < kTW; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) sm += fast_exp2(x[i][j] - m_use);
        sm = xgroup_sum(sm);
        if (g == 0) wpart[t][wave][n] = float2{mx, sm};
        if constexpr (kQT == 1) {                     // plain decode keeps the logits for part 2
#pragma unroll
            for (int i = 0; i < kTW; ++i)
                if (n < G && jw + 16 * i < n_vis[0])
                    *reinterpret_cast<float4 *>(zbuf + (((int64_t)b * dm.Hkv + h) * G + n) * n_c_cap + jw + 16 * i + 4 * g) =
                        float4{x[i][0], x[i][1], x[i][2], x[i][3]};
        }
    }
    __syncthreads();
    if (threadIdx.x < 16 * kQT) {                     // merge the four waves: one partial per head and query
        const int t = threadIdx.x >> 4, head = threadIdx.x & 15;
        if (head < G && qi0 + t < dm.n_q) {
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) M = fmaxf(M, wpart[t][w][head].x);
            const float mu = M == -INFINITY ? 0.f : M;
            float S = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) S += wpart[t][w][head].y * fast_exp2(wpart[t][w][head].x - mu);
            const int64_t bv = (int64_t)b * dm.n_q + qi0 + t;
            part[((bv * dm.Hkv + h) * G + head) * n_part + blockIdx.x] = float2{M, S};
        }
    }
    // Approximate log-sum-exp ("Efficient Top-K Implementation", last paragraph): the same
    // partial (max, sum) over the coarse kernels kChunk/rho * bx .. of this chunk, each the bf16 mean
    // of its rho fine kernels rho*c + 2r (exact sum in fp64, one rounding).
    if (dm.rho > 1) {                                 // uniform over the launch
        const int tiles_c = 4 * kTW / dm.rho;         // 16-kernel tiles of coarse kernels per workgroup
        const int n_vis_c_max = num_coarse(n_vis_max, dm.rho);
        float Mc[kQT], Sc[kQT];                       // running partial of this wave, reduced over the wave
#pragma unroll
        for (int t = 0; t < kQT; ++t) {
            Mc[t] = -INFINITY;
            Sc[t] = 0.f;
        }
        for (int tc = wave; tc < tiles_c; tc += 4) {
            const int c0 = blockIdx.x * (kChunk / dm.rho) + tc * 16, cc = c0 + n;
            bf16x8 ac[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                ac[ks] = zero8();
                if (cc < n_vis_c_max) {
                    double acc[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] = 0.0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (r >= dm.rho) break;
                        const int jf = dm.rho * cc + 2 * r;
                        bf16x8 v;
                        if (kAppend && closes && jf == n_vis_max - 1)
                            // the kernel this step completes: another workgroup may be storing it right now,
                            // so its row is built here from the cache and the new key, never read back
                            v = fresh_kernel_row8(ap, b, h, L_all, 32 * ks + 8 * g);
                        else
                            v = load8(ck.ptr + b * ck.sb + h * ck.sh + (int64_t)jf * ck.st + 32 * ks + 8 * g);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[e] += (double)(float)v[e];
                    }
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        w[e] = (uint32_t)f64_to_bf16_rne(acc[2 * e] / (double)dm.rho) |
                               ((uint32_t)f64_to_bf16_rne(acc[2 * e + 1] / (double)dm.rho) << 16);
                    ac[ks] = __builtin_bit_cast(bf16x8, uint4{w[0], w[1], w[2], w[3]});
                }
            }
#pragma unroll
            for (int t = 0; t < kQT; ++t) {
                const int n_vis_c = num_coarse(n_vis[t], dm.rho);
                f32x4 zc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) zc = mfma16(ac[ks], bq[t][ks], zc);
                float mc = -INFINITY, xc[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    xc[j] = c0 + 4 * g + j < n_vis_c ? zc[j] * dm.scale_log2 : -INFINITY;
                    mc = fmaxf(mc, xc[j]);
                }
                mc = xgroup_max(mc);
                const float Mn = fmaxf(Mc[t], mc), mu = Mn == -INFINITY ? 0.f : Mn;
                float sc = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) sc += fast_exp2(xc[j] - mu);
                sc = xgroup_sum(sc);
                Sc[t] = Sc[t] * fast_exp2(Mc[t] - mu) + sc;
                Mc[t] = Mn;
            }
        }
#pragma unroll
        for (int t = 0; t < kQT; ++t)
            if (g == 0) wpart_c[t][wave][n] = float2{Mc[t], Sc[t]};
        __syncthreads();
        if (threadIdx.x < 16 * kQT) {
            const int t = threadIdx.x >> 4, head = threadIdx.x & 15;
            if (head < G && qi0 + t < dm.n_q) {
                float M = -INFINITY;
#pragma unroll
                for (int w = 0; w < 4; ++w) M = fmaxf(M, wpart_c[t][w][head].x);
                const float mu = M == -INFINITY ? 0.f : M;
                float S = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) S += wpart_c[t][w][head].y * fast_exp2(wpart_c[t][w][head].x - mu);
                const int64_t bv = (int64_t)b * dm.n_q + qi0 + t;
                part_c[((bv * dm.Hkv + h) * G + head) * n_part + blockIdx.x] = float2{M, S};
            }
        }
    }
}

// ---- part 2, several queries per sequence: block scores ----------------------------------------------
// grid (nb_cap / (16*kTW), Hkv, B * ceil(n_q/kQT)), 256 threads (every block has a workgroup, also a
// last one too short to hold a complete kernel).  Workgroup bx pools blocks
// 16*kTW*bx .. +16*kTW-1 of kQT consecutive query tokens; block j needs kernels 4j-1 .. 4j+3, so the
// workgroup scores 4*kTW+1 tiles of 16 kernels starting one tile before its chunk (of that halo tile
// only the last kernel is used).  The logits are computed again rather than kept from part 1: a
// kernel's output has to reach memory before the next kernel starts, and megabytes of logits per
// query cost more than the matrix-core work to redo them.
// Z = Q . CK^T: lane = kernel (column), 4 accumulator entries = 4 consecutive heads.  A lane adds its 4
// heads; the four 16-lane groups leave their sums side by side in LDS and the pooling adds them, so
// no cross-lane traffic sits between the matrix cores and the scores.
template <int kQT>
__global__ __launch_bounds__(256) void decode_scores_kernel(Dims dm, Tensor q, Tensor ck,
                                                             const int32_t *__restrict__ seqlens,
                                                             const float2 *__restrict__ part, int32_t n_part,
                                                             float *__restrict__ R, int32_t nb_cap) {
    constexpr int kTW = tiles_per_wave2(kQT), kChunk = 64 * kTW, kTiles = 4 * kTW + 1;
    constexpr int kChunk1 = 64 * tiles_per_wave(kQT);  // kernels per partial of part 1
    constexpr int kLanesPerPair = 256 / (16 * kQT);   // lanes that merge the partials of one (query, head)
    constexpr int kMaxPartsPerLane = 16384 / kChunk1 / kLanesPerPair;   // contexts up to 262144 tokens
    __shared__ __align__(16) float lse_h[kQT][16];
    __shared__ float rs[kQT][4][kTiles * 16];         // per 16-lane group: head sums of kernels chunk-16 .. chunk+kChunk-1
    __shared__ __align__(16) uint16_t qs[kQT > 1 ? kQT * 16 * kQsPitch : 8];
    const int h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int G = dm.G;
    const int n_qt = (dm.n_q + kQT - 1) / kQT;
    const int b = kQT == 1 ? blockIdx.z : blockIdx.z / n_qt;   // kQT = 1 is only launched with n_q = 1
    const int qi0 = (blockIdx.z - b * n_qt) * kQT;
    const int L_all = clamp_len(seqlens[b], dm.max_seqlen);
    int L_max = 0;
#pragma unroll
    for (int t = 0; t < kQT; ++t) L_max = max(L_max, row_len(dm, L_all, qi0 + t));
    if (L_max < 1 || (int)blockIdx.x * 16 * kTW > (L_max - 1) / kBlock) return;    // no block of this chunk exists
    const int n_vis_max = num_kernels(L_max);
    const int first = (int)blockIdx.x * kChunk - 16;  // kernel of rs[.][.][0]
    // ---- operand loads: this wave's kernel tiles (tile 0 is the halo, taken by wave 3), the query rows ----
    bf16x8 aq[kQT][4], bk[kTW + 1][4];
#pragma unroll
    for (int i = 0; i <= kTW; ++i) {
        const int tile = i < kTW ? 1 + wave * kTW + i : 0;
        const int jh = first + 16 * tile + n;
        const bool have = (i < kTW || wave == 3) && jh >= 0 && jh < n_vis_max;
        const __bf16 *ckr = ck.ptr + b * ck.sb + h * ck.sh + (int64_t)jh * ck.st + 8 * g;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bk[i][ks] = zero8();
            if (have) bk[i][ks] = load8(ckr + 32 * ks);
        }
    }
    // ---- log-sum-exp per (query, head): kLanesPerPair lanes each, all loads of a lane issued together ----
    {
        const int pair = tid / kLanesPerPair, sub = tid % kLanesPerPair;
        const int t = pair >> 4, head = pair & 15;
        const int np = (num_kernels(row_len(dm, L_all, qi0 + t)) + kChunk1 - 1) / kChunk1;   // valid partials
        const int64_t bv = (int64_t)b * dm.n_q + min(qi0 + t, dm.n_q - 1);
        const float2 *pr = part + ((bv * dm.Hkv + h) * G + min(head, G - 1)) * n_part;
        float2 v[kMaxPartsPerLane];
#pragma unroll
        for (int i = 0; i < kMaxPartsPerLane; ++i) {
            const int p = sub + kLanesPerPair * i;
            v[i] = float2{-INFINITY, 0.f};
            if (p < np) v[i] = pr[p];
        }
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < kMaxPartsPerLane; ++i) m = fmaxf(m, v[i].x);
#pragma unroll
        for (int o = 1; o < kLanesPerPair; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
        const float mu = m == -INFINITY ? 0.f : m;
        float sm = 0.f;
#pragma unroll
        for (int i = 0; i < kMaxPartsPerLane; ++i) sm += v[i].y * fast_exp2(v[i].x - mu);
#pragma unroll
        for (int o = 1; o < kLanesPerPair; o <<= 1) sm += __shfl_xor(sm, o);
        if (sub == 0)      // approximate mode: rho times fewer kernels were summed; 0 when none is visible
            lse_h[t][head] = dm.rho > 1 ? (m == -INFINITY ? 0.f : m + fast_log2(sm) + (float)(31 - __clz(dm.rho)))
                                        : m + fast_log2(sm);
    }
    load_query_operands<kQT>(dm, q, b, h, qi0, qs, aq);     // (a barrier inside when kQT > 1)
    __syncthreads();
    // ---- head sums of exp(z - lse) ------------------------------------------------------------------------
#pragma unroll
    for (int t = 0; t < kQT; ++t) {
        const float4 l4 = *reinterpret_cast<const float4 *>(&lse_h[t][4 * g]);
        const float lh[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
        for (int i = 0; i <= kTW; ++i) {
            if (i == kTW && wave != 3) break;         // uniform over the wave
            const int tile = i < kTW ? 1 + wave * kTW + i : 0;
            f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) z = mfma16(aq[t][ks], bk[i][ks], z);
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (4 * g + r < G) acc += fast_exp2(z[r] * dm.scale_log2 - lh[r]);
            rs[t][g][16 * tile + n] = acc;
        }
    }
    __syncthreads();
    // ---- group mean, clamps, 5/4 max-pool: thread (t, jl) takes kernels 4j-1 .. 4j+3 = rs[..][4*jl+15 .. +19] ----
    if (tid < kQT * 16 * kTW) {
        const int t = tid / (16 * kTW), jl = tid % (16 * kTW);
        const int j = blockIdx.x * 16 * kTW + jl;
        const int L = row_len(dm, L_all, qi0 + t);
        if (L >= 1 && j <= (L - 1) / kBlock) {
            const int n_vis = num_kernels(L);
            float v = -INFINITY;
#pragma unroll
            for (int x = 0; x < 5; ++x) {
                const int c = 4 * jl + 15 + x, jh = first + c;
                const float sum = (rs[t][0][c] + rs[t][1][c]) + (rs[t][2][c] + rs[t][3][c]);
                if (jh >= 0 && jh < n_vis) v = fmaxf(v, fminf(fmaxf(sum * (1.f / G), kScoreFloor), kScoreCeil));
            }
            const int64_t bv = (int64_t)b * dm.n_q + qi0 + t;
            R[(bv * dm.Hkv + h) * nb_cap + j] = v;
        }
    }
}

// ---- part 2, plain decode: block scores from the logits part 1 kept ---------------------------------
// (One query per sequence: its logits are a quarter of the bytes of the compressed keys, so reading
// them back is cheaper than computing them again; with several queries per sequence the balance tips.)
// grid (nb_cap/64, Hkv, B), 320 threads.  Thread t <= 256 scores kernel 256*bx - 1 + t
// (one halo kernel to the left); threads 0..63 then pool blocks 64*bx + t.
constexpr int kMaxParts = 128;                        // partials per head (of >= 128 kernels): contexts up to 262144 tokens
__global__ __launch_bounds__(320) void decode_scores_z_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                             const float *__restrict__ zbuf,
                                                             const float2 *__restrict__ part,
                                                             int32_t n_c_cap, int32_t n_part, int32_t part_kernels,
                                                             float *__restrict__ R, int32_t nb_cap) {
    __shared__ float lse_h[16];
    __shared__ float rs[260];
    const int h = blockIdx.y, bv = blockIdx.z;
    const int tid = threadIdx.x;
    const int G = dm.G;
    const int base = blockIdx.x * 256;
    // Everything this thread reads lies in the workspace at places that do not depend on the sequence
    // length, so the loads go out before the length is known (one memory round trip less on the
    // critical path of the step); what turns out to be past the end is masked afterwards.
    const int head = min(tid >> 4, G - 1), sub = tid & 15;
    float2 v[kMaxParts / 16];
#pragma unroll
    for (int i = 0; i < kMaxParts / 16; ++i)
        v[i] = part[(((int64_t)bv * dm.Hkv + h) * G + head) * n_part + min(sub + 16 * i, n_part - 1)];
    const int jh = base - 1 + tid;
    const int jh_c = min(max(jh, 0), n_c_cap - 1);
    float zz[16];
#pragma unroll
    for (int gq = 0; gq < 16; ++gq) zz[gq] = zbuf[(((int64_t)bv * dm.Hkv + h) * G + min(gq, G - 1)) * n_c_cap + jh_c];
    int b, qi;
    const int L = query_row(dm, seqlens, bv, b, qi);
    const int n_vis = num_kernels(L);
    if (L < 1 || (int)blockIdx.x * 64 > (L - 1) / kBlock) return;            // no block of this chunk exists
    const int np = (n_vis + part_kernels - 1) / part_kernels;   // valid partials
    // log-sum-exp per head: 16 lanes per head
    if (tid < 256) {
#pragma unroll
        for (int i = 0; i < kMaxParts / 16; ++i)
            if (sub + 16 * i >= np) v[i] = float2{-INFINITY, 0.f};
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < kMaxParts / 16; ++i) m = fmaxf(m, v[i].x);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
        const float mu = m == -INFINITY ? 0.f : m;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < kMaxParts / 16; ++i) s += v[i].y * fast_exp2(v[i].x - mu);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o);
        if (sub == 0 && (tid >> 4) < G)   // approximate mode: rho times fewer kernels were summed; 0 when none is visible
            lse_h[tid >> 4] = dm.rho > 1 ? (m == -INFINITY ? 0.f : m + fast_log2(s) + (float)(31 - __clz(dm.rho)))
                                         : m + fast_log2(s);
    }
    // logits of this thread's kernel, all heads
    const bool have = tid <= 256 && jh >= 0 && jh < n_vis;
    __syncthreads();
    if (tid <= 256) {
        float acc = 0.f;
#pragma unroll
        for (int gq = 0; gq < 16; ++gq)
            if (gq < G) acc += fast_exp2(zz[gq] - lse_h[gq]);
        rs[tid] = have ? fminf(fmaxf(acc * (1.f / G), kScoreFloor), kScoreCeil) : -INFINITY;
    }
    __syncthreads();
    if (tid < 64) {
        const int j = blockIdx.x * 64 + tid;          // kernels 4j-1 .. 4j+3 = rs[4*tid .. 4*tid+4]
        if (j <= (L - 1) / kBlock) {
            float v = rs[4 * tid];
#pragma unroll
            for (int x = 1; x < 5; ++x) v = fmaxf(v, rs[4 * tid + x]);
            R[((int64_t)bv * dm.Hkv + h) * nb_cap + j] = v;
        }
    }
}

// ---- selection, part 3: top-k of one row of block scores ----------------------------------------
// grid (B*n_q*Hkv), 256 threads.  Candidates are the blocks n_init .. b_own - n_local; the forced ones
// are added afterwards (section 2.1.2 "Top-K Blocks Sharing": initial and local blocks are always
// attended).  Scores are positive floats, so their bit patterns order like unsigned integers.
// An element is the 64-bit word  key << 32 | ~block  with key = bits of the score (1 for a block
// without visible kernel, -inf): larger word = better element, ties go to the lower block index,
// and no two elements are equal.  Words below 2^32 (key 0) are "not a candidate".
//
// No serial rounds (a dependent chain per pick is what makes a small top-k slow on this machine);
// filters by counting instead, every comparison independent of the others.  Thread t keeps blocks
// t, t+256, ... in registers and `best`, the largest of them.  An element of the final top-k can
// only sit in a thread whose best is among the n_pick largest thread maxima (every better thread
// holds an element that beats it), and it is at least tau, the n_pick-th largest thread maximum
// (the n_pick largest thread maxima are n_pick distinct elements).
//   1a. rank of `best` inside its wavefront; the n_pick best of each wavefront survive
//   1b. rank of the survivors among all survivors = rank among all thread maxima; gives tau
//   2.  the n_pick best threads publish their elements >= tau; rank by counting among those
constexpr int kPickThreads = 256, kPickMaxVPT = 16;
// LDS of the top-k, carved out of the kernel's dynamic shared memory (16-byte aligned) so that its size
// follows the call's top-k instead of the largest one supported.
template <int kThreads>
struct PickShared {
    uint64_t *tmax;                                       // [kThreads] thread maxima, 64 per wavefront
    uint64_t *top;                                        // [kWaves * topk + 4] per wavefront: its n_pick best (0 = none)
    uint64_t *cand;                                       // [kWaves][cand_cap] per wavefront: elements that can still make it
    int *picked;                                          // [topk]
    int cand_cap;
    __device__ PickShared(unsigned char *smem, int topk, int vpt) {
        tmax = reinterpret_cast<uint64_t *>(smem);
        top = tmax + kThreads;
        cand = top + ((kThreads / 64 * topk + 4 + 1) & ~1);
        cand_cap = (topk * vpt + 3) & ~3;
        picked = reinterpret_cast<int *>(cand + kThreads / 64 * cand_cap);
    }
};
static inline size_t pick_shared_bytes(int threads, int topk, int vpt) {
    const size_t words = (size_t)threads + (((size_t)threads / 64 * topk + 4 + 1) & ~(size_t)1) +
                         (size_t)threads / 64 * (((size_t)topk * vpt + 3) & ~(size_t)3);
    return words * sizeof(uint64_t) + (size_t)topk * sizeof(int);
}

// Top-k of one row of block scores for a query at cache row L - 1 (L >= 1), by a whole workgroup of
// kThreads threads; thread t passes the scores of blocks t, t + kThreads, ... in r.  The selected
// blocks, ascending, go to `o` (a row of the block_idx output, padded with -1; may be null) and to
// `sel` (LDS, may be null).  Returns their number.  Contains barriers: every thread calls it.
//
// Two levels.  Every wavefront finds the n_pick best of its own share on its own, synchronising with
// nobody: rank its 64 thread maxima by counting; an element of its top n_pick can only sit in a
// thread whose maximum is among the n_pick largest, and is at least tau, the n_pick-th largest
// maximum; those threads publish their elements >= tau (a handful) and the wavefront ranks them by
// counting.  After one workgroup barrier the (at most) kWaves * n_pick finalists are ranked the same
// way.  A step that waits for the slowest wavefront costs more here than the arithmetic between two
// of them, hence as few of those as possible.
template <int kThreads, int kVPT>
__device__ inline int pick_row(const Dims &dm, int L, const float (&r)[kVPT], const PickShared<kThreads> &sh,
                               int32_t *__restrict__ o, int *sel) {
    constexpr int kWaves = kThreads / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b_own = (L - 1) / kBlock, n_blk = b_own + 1;
    const int n_sel = dm.topk < n_blk ? dm.topk : n_blk;
    const int n_init = dm.n_init < n_blk ? dm.n_init : n_blk;                 // forced leading blocks
    const int lo_local = max(n_init, b_own - dm.n_local + 1);                 // forced trailing: lo_local..b_own
    const int jc_max = lo_local - 1;                                          // candidates: n_init..jc_max
    const int n_pick = n_sel - (n_init + (b_own - lo_local + 1));
    if (n_pick > 0) {                                                         // uniform over the workgroup
        const int n_top = (kWaves * n_pick + 3) & ~3;
        uint64_t *wtop = sh.top + wave * n_pick, *wcand = sh.cand + wave * sh.cand_cap, *wmax = sh.tmax + 64 * wave;
        if (lane < n_pick) wtop[lane] = 0ull;
        if (wave == kWaves - 1 && lane < n_top - kWaves * n_pick) sh.top[kWaves * n_pick + lane] = 0ull;
        uint64_t el[kVPT], best = 0ull;
#pragma unroll
        for (int s = 0; s < kVPT; ++s) {
            const int j = tid + kThreads * s;
            const uint32_t kj = r[s] == -INFINITY ? 1u : __float_as_uint(r[s]);
            const uint32_t key = (j >= n_init && j <= jc_max) ? kj : 0u;
            el[s] = ((uint64_t)key << 32) | (uint32_t)~j;
            best = el[s] > best ? el[s] : best;
        }
        const bool real = best >= kPickValid;
        wmax[lane] = best;
        __builtin_amdgcn_wave_barrier();                  // same wavefront: LDS keeps the order
        const int lrank = count_larger(wmax, 64, best);
        const bool finalist = real && lrank < n_pick;
        uint64_t tau = kPickValid;                        // the n_pick-th largest maximum, if there are that many real ones
        const uint64_t who = __ballot(real && lrank == n_pick - 1);
        if (who) {
            const int src = __builtin_ctzll(who);
            tau = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(best >> 32), src) << 32) |
                  (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)best, src);
        }
        int n_cand = 0;                                   // <= n_pick * kVPT <= cand_cap
        const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
        for (int s = 0; s < kVPT; ++s) {
            const bool pub = finalist && el[s] >= tau;
            const uint64_t m = __ballot(pub);
            if (pub) wcand[n_cand + __popcll(m & below)] = el[s];
            n_cand += __popcll(m);
        }
        const int n_cand4 = (n_cand + 3) & ~3;
        if (lane < n_cand4 - n_cand) wcand[n_cand + lane] = 0ull;
        __builtin_amdgcn_wave_barrier();
        for (int i = lane; i < n_cand; i += 64) {
            const uint64_t e = wcand[i];
            const int beaten = count_larger(wcand, n_cand4, e);
            if (beaten < n_pick) wtop[beaten] = e;
        }
        __syncthreads();
        if (tid < kWaves * n_pick) {                      // kWaves * n_pick <= kThreads: n_pick <= 64
            const uint64_t e = sh.top[tid];
            if (e >= kPickValid) {
                const int beaten = count_larger(sh.top, n_top, e);
                if (beaten < n_pick) sh.picked[beaten] = (int)~(uint32_t)e;
            }
        }
        __syncthreads();
    }
    if (wave == 0) {
        int mine = 0x7fffffff;
        if (lane < n_pick) mine = sh.picked[lane];
        else if (lane < n_sel) {
            const int f = lane - n_pick;
            mine = f < n_init ? f : lo_local + (f - n_init);
        }
        // ascending order: rank = number of selected blocks below mine
        int rank = 0;
        for (int e = 0; e < n_sel; ++e) rank += __builtin_amdgcn_readlane(mine, e) < mine ? 1 : 0;
        if (lane < n_sel) {
            if (o) o[rank] = mine;
            if (sel) sel[rank] = mine;
        } else if (o && lane < dm.topk) {
            o[lane] = -1;
        }
    }
    return n_sel;
}

template <int kVPT>
__global__ __launch_bounds__(kPickThreads) void decode_pick_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                                    const float *__restrict__ R, int32_t nb_cap,
                                                                    int32_t *__restrict__ block_idx) {
    extern __shared__ __align__(16) unsigned char pick_smem[];
    const PickShared<kPickThreads> sh(pick_smem, dm.topk, kVPT);
    const int row = blockIdx.x, bv = row / dm.Hkv, h = row - bv * dm.Hkv;
    const int tid = threadIdx.x;
    const float *Rr = R + (int64_t)row * nb_cap;
    float r[kVPT];                                        // every load issued before any use
#pragma unroll
    for (int s = 0; s < kVPT; ++s) r[s] = Rr[min(tid + kPickThreads * s, nb_cap - 1)];
    int b, qi;
    const int L = query_row(dm, seqlens, bv, b, qi);
    int32_t *o = block_idx + (((int64_t)b * dm.Hkv + h) * dm.n_q + qi) * dm.topk;
    if (L < 1) {
        if (tid < dm.topk) o[tid] = -1;
        return;
    }
    pick_row<kPickThreads, kVPT>(dm, L, r, sh, o, nullptr);
}

// ---- attention, part 1: one workgroup per selected block --------------------------------------
// grid (topk, Hkv, B), 256 threads.  Every load of the block (64 key rows as MFMA operands, 64
// value rows for LDS, the query) is issued before anything is used.  Wave w: S^T = K . Q^T for
// keys 16w..16w+15; the probabilities go to LDS as P[key][head]; then wave w owns value channels
// 32w..32w+31 and computes O^T = V^T . P^T on the matrix cores, gathering the V^T fragments
// (8 keys of one channel per lane) from the row-major value tile in LDS.
constexpr int kVsPitch = kHeadDim + 4;               // bf16 elements per LDS value row: conflict-free column reads
// Partial attention of query row bv = (b, qi), L cache rows up to and including the query, over
// selected block `blk` (entry cidx of the row's list; < 0: none).  Whole workgroup of 256 threads.
__device__ inline void attend_block(const Dims &dm, const Tensor &q, const Tensor &k, const Tensor &v, int bv, int b,
                                    int qi, int h, int cidx, int L, int blk, const uint64_t *__restrict__ tree_mask,
                                    float *__restrict__ o_part, float2 *__restrict__ ml_part) {
    __shared__ __align__(16) uint16_t Vs[kBlock * kVsPitch];
    __shared__ float Ps[kBlock][17];
    __shared__ float wmax[4][16], wsum[4][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int G = dm.G;
    const int L_all = L + (dm.n_q - 1 - qi);             // cache rows of the sequence (when L >= 1)
    uint64_t mask_word = 0ull;
    if (tree_mask) mask_word = tree_mask[bv];
    // a tree mask may let a query attend drafted tokens that lie after it in the cache
    const bool valid = L >= 1 && blk >= 0 && (int64_t)blk * kBlock < (tree_mask ? L_all : L);
    if (!valid) {                                        // uniform over the workgroup
        const int head = tid & 15, chunk = tid >> 4;
        if (head < G) {
            const int64_t pbase = (((int64_t)bv * dm.Hq + h * G + head) * dm.topk + cidx);
            if (chunk == 0) ml_part[pbase] = float2{-INFINITY, 0.f};
            float4 zf = {0.f, 0.f, 0.f, 0.f};
            float4 *op = reinterpret_cast<float4 *>(o_part + pbase * kHeadDim + 8 * chunk);
            op[0] = zf;
            op[1] = zf;
        }
        return;
    }
    const int key0 = blk * kBlock;
    const int last_row = dm.max_seqlen - 1;              // rows the query may not see are read (in bounds) and masked
    // ---- all loads --------------------------------------------------------------------------------
    const int c8 = tid & 15, vr = tid >> 4;
    uint4 vrow[4];
    {
        const __bf16 *vb = v.ptr + b * v.sb + h * v.sh + 8 * c8;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            vrow[i] = *reinterpret_cast<const uint4 *>(vb + (int64_t)min(key0 + vr + 16 * i, last_row) * v.st);
    }
    bf16x8 a[4], bq[4];
    {
        const int key = min(key0 + 16 * wave + n, last_row);
        const __bf16 *kr = k.ptr + b * k.sb + h * k.sh + (int64_t)key * k.st + 8 * g;
        const __bf16 *qr = q.ptr + b * q.sb + qi * q.st + (int64_t)(h * G + min(n, G - 1)) * q.sh + 8 * g;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            a[ks] = load8(kr + 32 * ks);
            bq[ks] = load8(qr + 32 * ks);
        }
    }
    // ---- which of the block's 64 keys the query attends: bit r = key key0 + r ------------------------
    // Causal: keys up to the query's own position.  Tree mask: every context key (before the drafted
    // tokens), and drafted token j iff bit j of the query's mask word is set.
    uint64_t allow;
    if (!tree_mask) {
        const int nv = L - key0;                         // >= 1
        allow = nv >= 64 ? ~0ull : (1ull << nv) - 1ull;
    } else {
        const int l_ctx = L_all - dm.n_q;                // >= 0
        const uint64_t mw = dm.n_q >= 64 ? mask_word : mask_word & ((1ull << dm.n_q) - 1ull);
        const int sh = key0 - l_ctx;                     // block offset of the first drafted token, negated
        if (sh >= 0) allow = sh < 64 ? mw >> sh : 0ull;
        else allow = sh > -64 ? (mw << -sh) | ((1ull << -sh) - 1ull) : ~0ull;
    }
    // ---- value tile to LDS (masked rows as zeros: 0 * garbage must stay 0) ----------------------------
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = vr + 16 * i;
        uint4 x = vrow[i];
        if (!((allow >> r) & 1ull)) x = uint4{0u, 0u, 0u, 0u};
        *reinterpret_cast<uint2 *>(&Vs[r * kVsPitch + 8 * c8]) = uint2{x.x, x.y};
        *reinterpret_cast<uint2 *>(&Vs[r * kVsPitch + 8 * c8 + 4]) = uint2{x.z, x.w};
    }
    // ---- scores of this wave's 16 keys ---------------------------------------------------------------
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) s = mfma16(a[ks], bq[ks], s);
    float x[4], mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[j] = ((allow >> (16 * wave + 4 * g + j)) & 1ull) ? s[j] * dm.scale_log2 : -INFINITY;
        mx = fmaxf(mx, x[j]);
    }
    mx = xgroup_max(mx);
    if (g == 0) wmax[wave][n] = mx;
    __syncthreads();
    const float m = fmaxf(fmaxf(wmax[0][n], wmax[1][n]), fmaxf(wmax[2][n], wmax[3][n]));
    const float m_sub = m == -INFINITY ? 0.f : m;       // -inf only when a tree mask hides the whole block
    float ps = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float p = fast_exp2(x[j] - m_sub);
        ps += p;
        Ps[16 * wave + 4 * g + j][n] = p;
    }
    ps = xgroup_sum(ps);
    if (g == 0) wsum[wave][n] = ps;
    __syncthreads();
    // ---- O^T[channel, head] for channels 32*wave .. 32*wave+31 ---------------------------------------
    f32x4 o[2];
    o[0] = o[1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        bf16x8 pb;                                       // B: head n, keys 32kk + 8g .. +7
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)Ps[32 * kk + 8 * g + e][n];
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
            const uint16_t *vc = &Vs[(32 * kk + 8 * g) * kVsPitch + 32 * wave + 16 * ct + n];   // A: channel row n
            uint32_t w[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2)
                w[e2] = (uint32_t)vc[(2 * e2) * kVsPitch] | ((uint32_t)vc[(2 * e2 + 1) * kVsPitch] << 16);
            const uint4 av = {w[0], w[1], w[2], w[3]};
            o[ct] = mfma16(__builtin_bit_cast(bf16x8, av), pb, o[ct]);
        }
    }
    if (n < G) {                                         // lane: head n, channels 32w + 16ct + 4g .. +3
        const int64_t pbase = (((int64_t)bv * dm.Hq + h * G + n) * dm.topk + cidx);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
            *reinterpret_cast<float4 *>(o_part + pbase * kHeadDim + 32 * wave + 16 * ct + 4 * g) =
                float4{o[ct][0], o[ct][1], o[ct][2], o[ct][3]};
        if (wave == 0 && g == 0)
            ml_part[pbase] = float2{m, (wsum[0][n] + wsum[1][n]) + (wsum[2][n] + wsum[3][n])};
    }
}

__global__ __launch_bounds__(256) void decode_attn_partial_kernel(Dims dm, Tensor q, Tensor k, Tensor v,
                                                                   const int32_t *__restrict__ seqlens,
                                                                   const int32_t *__restrict__ block_idx,
                                                                   const uint64_t *__restrict__ tree_mask,
                                                                   float *__restrict__ o_part,
                                                                   float2 *__restrict__ ml_part) {
    const int cidx = blockIdx.x, h = blockIdx.y, bv = blockIdx.z;
    int b, qi;
    const int L = query_row(dm, seqlens, bv, b, qi);
    const int blk = block_idx[(((int64_t)b * dm.Hkv + h) * dm.n_q + qi) * dm.topk + cidx];
    attend_block(dm, q, k, v, bv, b, qi, h, cidx, L, blk, tree_mask, o_part, ml_part);
}

// Top-k and partial attention in one launch (the one-call decode and verification steps): a step is
// a chain of dependent launches, each costing a launch gap and a memory round trip, and the block
// list is the only thing the attention waits for.  Every one of the k workgroups of a (query row,
// key-value head) repeats the top-k on the same row of block scores (same result; workgroup 0 writes
// it out) and goes on with its own entry of the list.
template <int kVPT>
__global__ __launch_bounds__(kPickThreads) void decode_pick_partial_kernel(Dims dm, Tensor q, Tensor k, Tensor v,
                                                                            const int32_t *__restrict__ seqlens,
                                                                            const float *__restrict__ R, int32_t nb_cap,
                                                                            const uint64_t *__restrict__ tree_mask,
                                                                            int32_t *__restrict__ block_idx,
                                                                            float *__restrict__ o_part,
                                                                            float2 *__restrict__ ml_part) {
    extern __shared__ __align__(16) unsigned char pick_smem[];
    const PickShared<kPickThreads> sh(pick_smem, dm.topk, kVPT);
    __shared__ int sel[kMaxTopk];
    const int cidx = blockIdx.x, h = blockIdx.y, bv = blockIdx.z;
    const int tid = threadIdx.x;
    const float *Rr = R + ((int64_t)bv * dm.Hkv + h) * nb_cap;
    float r[kVPT];                                        // every load issued before any use
#pragma unroll
    for (int s = 0; s < kVPT; ++s) r[s] = Rr[min(tid + kPickThreads * s, nb_cap - 1)];
    int b, qi;
    const int L = query_row(dm, seqlens, bv, b, qi);
    int32_t *orow = block_idx + (((int64_t)b * dm.Hkv + h) * dm.n_q + qi) * dm.topk;
    int blk = -1;
    if (L < 1) {                                          // uniform over the workgroup
        if (cidx == 0 && tid < dm.topk) orow[tid] = -1;
    } else {
        const int n_sel = pick_row<kPickThreads, kVPT>(dm, L, r, sh, cidx == 0 ? orow : nullptr, sel);
        __syncthreads();
        if (cidx < n_sel) blk = sel[cidx];
    }
    attend_block(dm, q, k, v, bv, b, qi, h, cidx, L, blk, tree_mask, o_part, ml_part);
}

// ---- attention, part 2: merge the k partials of every query head ---------------------------------
// grid (Hq, B*n_q), 128 threads: thread = channel.  All partial loads are issued before the merge.
__global__ __launch_bounds__(128) void decode_merge_kernel(Dims dm, const float *__restrict__ o_part,
                                                            const float2 *__restrict__ ml_part, Tensor out,
                                                            float *__restrict__ lse) {
    const int hq = blockIdx.x, bv = blockIdx.y, cch = threadIdx.x;
    const int b = bv / dm.n_q, qi = bv - b * dm.n_q;
    const int64_t pbase = ((int64_t)bv * dm.Hq + hq) * dm.topk;
    float2 ml[kMaxTopk];
    float ov[kMaxTopk];
#pragma unroll
    for (int c = 0; c < kMaxTopk; ++c) {
        ml[c] = float2{-INFINITY, 0.f};
        ov[c] = 0.f;
        if (c < dm.topk) {
            ml[c] = ml_part[pbase + c];
            ov[c] = o_part[(pbase + c) * kHeadDim + cch];
        }
    }
    float M = -INFINITY;
#pragma unroll
    for (int c = 0; c < kMaxTopk; ++c) M = fmaxf(M, ml[c].x);
    float num = 0.f, den = 0.f;
    if (M > -INFINITY) {
#pragma unroll
        for (int c = 0; c < kMaxTopk; ++c) {
            const float w = fast_exp2(ml[c].x - M);
            den += w * ml[c].y;
            num += w * ov[c];
        }
    }
    const float o = den > 0.f ? num / den : 0.f;
    out.ptr[b * out.sb + qi * out.st + (int64_t)hq * out.sh + cch] = (__bf16)o;
    if (cch == 0) lse[(int64_t)bv * dm.Hq + hq] = den > 0.f ? (M + fast_log2(den)) * kLn2 : -INFINITY;
}

// ---- host side -------------------------------------------------------------------------------------
static inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

struct DecodeSelLayout {
    int32_t n_c_cap, n_part, nb_cap;
    size_t z_bytes, part_bytes, r_bytes;              // z: logits, plain decode only
};
static DecodeSelLayout decode_sel_layout(const Dims &dm) {
    DecodeSelLayout l;
    int32_t n_c = num_kernels(dm.max_seqlen);
    l.n_c_cap = (n_c + 255) / 256 * 256;
    if (l.n_c_cap < 256) l.n_c_cap = 256;
    l.n_part = l.n_c_cap / (64 * (dm.n_q == 1 ? decode_tiles_per_wave(dm) : tiles_per_wave(kVerifyQT)));
    l.nb_cap = ((dm.max_seqlen + kBlock - 1) / kBlock + 63) / 64 * 64;
    const size_t rows = (size_t)dm.batch * dm.n_q;
    l.z_bytes = dm.n_q == 1 ? align256(rows * dm.Hq * l.n_c_cap * sizeof(float)) : 0;
    l.part_bytes = align256(rows * dm.Hq * l.n_part * sizeof(float2));
    l.r_bytes = align256(rows * dm.Hkv * l.nb_cap * sizeof(float));
    return l;
}

size_t select_decode_ws_bytes(const Dims &dm) {
    DecodeSelLayout l = decode_sel_layout(dm);
    return l.z_bytes + 2 * l.part_bytes + l.r_bytes;
}

int launch_select_decode(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                         int32_t *block_idx, void *ws, hipStream_t stream, const AppendArgs *append,
                         AttendArgs *attend) {
    if (dm.batch <= 0) return 0;
    DecodeSelLayout l = decode_sel_layout(dm);
    if (l.n_c_cap > 16384) return (int)hipErrorInvalidValue;         // rejected earlier by the C ABI
    char *wsb = reinterpret_cast<char *>(ws);
    float *zbuf = reinterpret_cast<float *>(wsb);
    float2 *part = reinterpret_cast<float2 *>(wsb + l.z_bytes);
    float2 *part_c = reinterpret_cast<float2 *>(wsb + l.z_bytes + l.part_bytes);
    float *R = reinterpret_cast<float *>(wsb + l.z_bytes + 2 * l.part_bytes);
    const int rows = dm.batch * dm.n_q;                              // <= 65535, checked by the C ABI
    const int n_qt = (dm.n_q + kVerifyQT - 1) / kVerifyQT;
    const float2 *part_lse = dm.rho > 1 ? part_c : part;
    timing_begin("decode_logits_kernel", stream);
    const AppendArgs no_append = {q, q, q, q};                       // unused placeholders
    const bool tw4 = decode_tiles_per_wave(dm) == 4;
    const dim3 grid1(l.n_part, dm.Hkv, dm.batch);
#define INFLLMV2_LOGITS(APPEND, TW, ARG)                                                                        \
    hipLaunchKernelGGL((decode_logits_kernel<1, APPEND, TW>), grid1, dim3(256), 0, stream, dm, q, ck, seqlens, \
                       zbuf, l.n_c_cap, part, part_c, l.n_part, ARG)
    if (dm.n_q == 1 && append) {
        if (tw4) INFLLMV2_LOGITS(true, 4, *append);
        else INFLLMV2_LOGITS(true, 2, *append);
    } else if (dm.n_q == 1) {
        if (tw4) INFLLMV2_LOGITS(false, 4, no_append);
        else INFLLMV2_LOGITS(false, 2, no_append);
    } else {
        hipLaunchKernelGGL((decode_logits_kernel<kVerifyQT, false, tiles_per_wave(kVerifyQT)>),
                           dim3(l.n_part, dm.Hkv, dm.batch * n_qt), dim3(256), 0, stream, dm, q, ck, seqlens, nullptr, 0,
                           part, part_c, l.n_part, no_append);
    }
#undef INFLLMV2_LOGITS
    timing_end(stream);
    timing_begin("decode_scores_kernel", stream);
    if (dm.n_q == 1)
        hipLaunchKernelGGL(decode_scores_z_kernel, dim3(l.nb_cap / 64, dm.Hkv, dm.batch), dim3(320), 0, stream,
                           dm, seqlens, zbuf, part_lse, l.n_c_cap, l.n_part, 64 * decode_tiles_per_wave(dm), R, l.nb_cap);
    else
        hipLaunchKernelGGL(decode_scores_kernel<kVerifyQT>,
                           dim3(l.nb_cap / (16 * tiles_per_wave2(kVerifyQT)), dm.Hkv, dm.batch * n_qt), dim3(256), 0,
                           stream, dm, q, ck, seqlens, part_lse, l.n_part, R, l.nb_cap);
    timing_end(stream);
    const int n_blocks = (dm.max_seqlen + kBlock - 1) / kBlock;
    if (n_blocks > kPickThreads * kPickMaxVPT) return (int)hipErrorInvalidValue;   // rejected earlier by the C ABI
    // Top-k and partial attention in one launch: every workgroup of the attention repeats the top-k of its
    // row, which is free while compute units idle and costs throughput once the launch fills the machine.
    constexpr int64_t kMaxFusedUnits = 1024;                         // (row, key-value head, block) workgroups
    if (attend) attend->fused = (int64_t)rows * dm.Hkv * dm.topk <= kMaxFusedUnits;
    if (attend && attend->fused) {
        const dim3 grid(dm.topk, dm.Hkv, rows), block(kPickThreads);
        timing_begin("decode_pick_partial_kernel", stream);
#define INFLLMV2_PICK_PARTIAL(VPT)                                                                                  \
    hipLaunchKernelGGL(decode_pick_partial_kernel<VPT>, grid, block, pick_shared_bytes(kPickThreads, dm.topk, VPT), \
                       stream, dm, q, attend->k, attend->v, seqlens, R, l.nb_cap, attend->tree_mask, block_idx,     \
                       attend->o_part, attend->ml_part)
        if (n_blocks <= kPickThreads * 4) INFLLMV2_PICK_PARTIAL(4);
        else if (n_blocks <= kPickThreads * 8) INFLLMV2_PICK_PARTIAL(8);
        else if (n_blocks <= kPickThreads * 12) INFLLMV2_PICK_PARTIAL(12);
        else INFLLMV2_PICK_PARTIAL(16);
#undef INFLLMV2_PICK_PARTIAL
        timing_end(stream);
        return (int)hipGetLastError();
    }
    const dim3 grid(rows * dm.Hkv), block(kPickThreads);
    timing_begin("decode_pick_kernel", stream);
    if (n_blocks <= kPickThreads * 4)
        hipLaunchKernelGGL(decode_pick_kernel<4>, grid, block, pick_shared_bytes(kPickThreads, dm.topk, 4), stream, dm,
                           seqlens, R, l.nb_cap, block_idx);
    else if (n_blocks <= kPickThreads * 8)
        hipLaunchKernelGGL(decode_pick_kernel<8>, grid, block, pick_shared_bytes(kPickThreads, dm.topk, 8), stream, dm,
                           seqlens, R, l.nb_cap, block_idx);
    else if (n_blocks <= kPickThreads * 12)
        hipLaunchKernelGGL(decode_pick_kernel<12>, grid, block, pick_shared_bytes(kPickThreads, dm.topk, 12), stream, dm,
                           seqlens, R, l.nb_cap, block_idx);
    else
        hipLaunchKernelGGL(decode_pick_kernel<16>, grid, block, pick_shared_bytes(kPickThreads, dm.topk, 16), stream, dm,
                           seqlens, R, l.nb_cap, block_idx);
    timing_end(stream);
    return (int)hipGetLastError();
}

size_t attn_decode_ws_bytes(const Dims &dm) {
    const size_t o = align256((size_t)dm.batch * dm.n_q * dm.Hq * dm.topk * kHeadDim * sizeof(float));
    const size_t ml = align256((size_t)dm.batch * dm.n_q * dm.Hq * dm.topk * sizeof(float2));
    return o + ml;
}

static void attn_decode_ws(const Dims &dm, void *ws, float *&o_part, float2 *&ml_part) {
    const size_t o_bytes = align256((size_t)dm.batch * dm.n_q * dm.Hq * dm.topk * kHeadDim * sizeof(float));
    o_part = reinterpret_cast<float *>(ws);
    ml_part = reinterpret_cast<float2 *>(reinterpret_cast<char *>(ws) + o_bytes);
}

static void launch_decode_partial(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                                  const int32_t *block_idx, const uint64_t *tree_mask, float *o_part, float2 *ml_part,
                                  hipStream_t stream) {
    timing_begin("decode_attn_partial_kernel", stream);
    hipLaunchKernelGGL(decode_attn_partial_kernel, dim3(dm.topk, dm.Hkv, dm.batch * dm.n_q), dim3(256), 0, stream,
                       dm, q, k, v, seqlens, block_idx, tree_mask, o_part, ml_part);
    timing_end(stream);
}

static int launch_decode_merge(const Dims &dm, const float *o_part, const float2 *ml_part, Tensor out, float *lse,
                               hipStream_t stream) {
    timing_begin("decode_merge_kernel", stream);
    hipLaunchKernelGGL(decode_merge_kernel, dim3(dm.Hq, dm.batch * dm.n_q), dim3(128), 0, stream, dm, o_part,
                       ml_part, out, lse);
    timing_end(stream);
    return (int)hipGetLastError();
}

int launch_attn_decode(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                       const int32_t *block_idx, const uint64_t *tree_mask, Tensor out, float *lse, void *ws,
                       hipStream_t stream) {
    if (dm.batch <= 0) return 0;
    float *o_part;
    float2 *ml_part;
    attn_decode_ws(dm, ws, o_part, ml_part);
    launch_decode_partial(dm, q, k, v, seqlens, block_idx, tree_mask, o_part, ml_part, stream);
    return launch_decode_merge(dm, o_part, ml_part, out, lse, stream);
}

// One decode step for one query per sequence: cache append + selection + attention, four launches.
int launch_decode_step(const Dims &dm, Tensor q, Tensor ck, const AppendArgs &append, const int32_t *seqlens,
                       int32_t *block_idx, Tensor out, float *lse, void *ws_select, void *ws_attn,
                       hipStream_t stream) {
    if (dm.batch <= 0) return 0;
    AttendArgs at = {append.k, append.v, nullptr, false, nullptr, nullptr};
    attn_decode_ws(dm, ws_attn, at.o_part, at.ml_part);
    const int err = launch_select_decode(dm, q, ck, seqlens, block_idx, ws_select, stream, &append, &at);
    if (err) return err;
    if (!at.fused) launch_decode_partial(dm, q, append.k, append.v, seqlens, block_idx, nullptr, at.o_part, at.ml_part, stream);
    return launch_decode_merge(dm, at.o_part, at.ml_part, out, lse, stream);
}

// One verification step for n_q drafted tokens per sequence: append (+ completed semantic kernels),
// selection per drafted token, tree-masked attention; five launches.
int launch_verify_step(const Dims &dm, Tensor q, Tensor ck, const AppendArgs &append, const int32_t *seqlens,
                       const uint64_t *tree_mask, int32_t *block_idx, Tensor out, float *lse, void *ws_select,
                       void *ws_attn, hipStream_t stream) {
    if (dm.batch <= 0) return 0;
    int err = launch_append_kv(dm, append.k_new, append.v_new, append.k, append.v, &ck, seqlens, stream);
    if (err) return err;
    AttendArgs at = {append.k, append.v, tree_mask, false, nullptr, nullptr};
    attn_decode_ws(dm, ws_attn, at.o_part, at.ml_part);
    err = launch_select_decode(dm, q, ck, seqlens, block_idx, ws_select, stream, nullptr, &at);
    if (err) return err;
    if (!at.fused) launch_decode_partial(dm, q, append.k, append.v, seqlens, block_idx, tree_mask, at.o_part, at.ml_part, stream);
    return launch_decode_merge(dm, at.o_part, at.ml_part, out, lse, stream);
}

}  // namespace infllmv2
