// Backward of the stage-3 attention (section 2.1: the sparse attention is trainable).  The block
// sets are a discrete choice and the mean-pooled semantic kernels have no parameters, so the
// gradient reaches q, k and v through the attention alone.  With p = exp(z - lse) recomputed from
// the forward's log-sum-exp, D = <dout, out> per (token, head):
//     dv_t += p dout_i        dp = <dout_i, v_t>        ds = p (dp - D)
//     dq_i += scale ds k_t    dk_t += scale ds q_i
//
// Per-token block sets make dq a gather (a token walks its blocks, like the forward) and dk/dv a
// scatter (a block collects from every token that selected it).  The scatter is turned around with
// a membership bitmap (block x token) built from the block lists, so both big kernels accumulate
// in registers:
//   bwd_prep_kernel     D, the exponent offsets -lse log2(e), and the membership bits of every token
//   pack_bwd_kernel     fragment-major copies of every block: K rows, V rows, K transposed
//   attn_bwd_dq_kernel  wavefront = 2 tokens, walks the union of their block lists:
//                       S^T = K.Q^T, dP^T = V.dO^T, dQ^T += K^T.dS^T
//   attn_bwd_dkdv_kernel  wavefront = 32 keys x 64 channels of a block, walks the member tokens of one
//                       segment in pairs: S = Q.K^T, dP = dO.V^T, dV^T += dO^T.P, dK^T += Q^T.dS
//                       (32x32x16 MFMAs; q and dout rows copied from memory straight into LDS);
//                       fp32 atomics merge the segments
//   bwd_finish_kernel   fp32 accumulators -> bf16 dk (times scale), dv
// As in the forward, every second contraction takes its B operand straight from the accumulator
// layout of the first, with the contraction index of the A fragments permuted to match.
#include "common.h"

namespace infllmv2 {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBwdBlockU4 = 3 * 16 * 64;              // uint4 per packed block: K rows, V rows, K^T (48 KiB)
// Member tokens of one dk/dv workgroup come from one segment of the sequence.  Short segments give
// more workgroups (better balance at 32K tokens), long ones fewer prologues and merges per block
// (at 128K tokens most (block, segment) units hold a handful of members).
static inline int bwd_seg_tokens(const Dims &dm) { return dm.max_seqlen > 65536 ? 8192 : 2048; }
constexpr int kBwdNone = 0x7fffffff;
constexpr int kBwdBlkBits = 27, kBwdBlkMask = (1 << kBwdBlkBits) - 1;

struct BwdLayout {
    int32_t nb_cap, words;                            // blocks per sequence; bitmap words per block row (multiple of 64)
    size_t kvb, delta, rowc, bitmap, acc_dk, acc_dv, total; // byte offsets into the workspace
    size_t zero_begin, zero_bytes;                    // the part that has to start at zero (bitmap and accumulators)
};
static inline size_t al256(size_t x) { return (x + 255) / 256 * 256; }
static BwdLayout bwd_layout(const Dims &dm) {
    BwdLayout l;
    const size_t T = (size_t)dm.max_seqlen, BH = (size_t)dm.batch * dm.Hkv;
    l.nb_cap = (dm.max_seqlen + kBlock - 1) / kBlock;
    const int seg_tokens = bwd_seg_tokens(dm);
    l.words = ((dm.max_seqlen + seg_tokens - 1) / seg_tokens) * (seg_tokens / 32);
    size_t o = 0;
    l.kvb = o;    o += al256(BH * l.nb_cap * kBwdBlockU4 * sizeof(uint4));
    l.delta = o;  o += al256((size_t)dm.batch * T * dm.Hq * sizeof(float));
    l.rowc = o;   o += al256((size_t)dm.batch * T * dm.Hkv * 32 * sizeof(float));
    l.zero_begin = o;
    l.bitmap = o; o += al256(BH * l.nb_cap * l.words * sizeof(uint32_t));
    l.acc_dk = o; o += al256(BH * T * kHeadDim * sizeof(float));
    l.acc_dv = o; o += al256(BH * T * kHeadDim * sizeof(float));
    l.zero_bytes = o - l.zero_begin;
    l.total = o;
    return l;
}

size_t attn_bwd_ws_bytes(const Dims &dm) { return bwd_layout(dm).total; }

__device__ inline int seq_len(const Dims &dm, const int32_t *__restrict__ seqlens, int b) {
    const int32_t L = seqlens[b];
    return L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
}

__global__ __launch_bounds__(256) void bwd_zero_kernel(uint4 *__restrict__ p, size_t n) {
    const uint4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = z;
}

// ---- per token: D and membership bits -----------------------------------------------------------------
// grid (ceil(T/4), Hkv, B); wave w handles token 4*bx + w for key-value head h.
__global__ __launch_bounds__(256) void bwd_prep_kernel(Dims dm, Tensor out, Tensor dout,
                                                        const int32_t *__restrict__ seqlens,
                                                        const int32_t *__restrict__ block_idx,
                                                        const float *__restrict__ lse, float *__restrict__ delta,
                                                        float *__restrict__ rowc, uint32_t *__restrict__ bitmap,
                                                        int32_t nb_cap, int32_t words) {
    const int h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tok = blockIdx.x * 4 + wave;
    const int L = seq_len(dm, seqlens, b);
    if (tok >= L) return;
    const int G = dm.G;
    const int row = lane >> 2, quarter = lane & 3;        // head of the group, 32 channels
    const int64_t ooff = b * out.sb + (int64_t)tok * out.st + (int64_t)(h * G + min(row, G - 1)) * out.sh + 32 * quarter;
    const int64_t goff = b * dout.sb + (int64_t)tok * dout.st + (int64_t)(h * G + min(row, G - 1)) * dout.sh + 32 * quarter;
    uint4 xo[4], xg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        xo[i] = *reinterpret_cast<const uint4 *>(out.ptr + ooff + 8 * i);
        xg[i] = *reinterpret_cast<const uint4 *>(dout.ptr + goff + 8 * i);
    }
    int blk = -1;
    if (lane < dm.topk) blk = block_idx[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * dm.topk + lane];
    float dsum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bf16x8 o8 = __builtin_bit_cast(bf16x8, xo[i]), g8 = __builtin_bit_cast(bf16x8, xg[i]);
#pragma unroll
        for (int e = 0; e < 8; ++e) dsum += (float)o8[e] * (float)g8[e];
    }
    dsum += __shfl_xor(dsum, 1);
    dsum += __shfl_xor(dsum, 2);
    if (quarter == 0 && row < G) delta[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + row] = dsum;
    // the same per (token, key-value head) as one 128-byte record for the dk/dv kernel: the exponent offsets
    // -lse log2(e) of the 16 head slots (-inf for slots past the group and for rows without a finite lse, whose
    // probabilities are then zero), then D
    if (quarter == 0) {
        float *rec = rowc + (((int64_t)b * dm.max_seqlen + tok) * dm.Hkv + h) * 32;
        float ne = -INFINITY;
        if (row < G) {
            const float ls = lse[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + row];
            if (ls > -INFINITY && ls < INFINITY) ne = -ls * kLog2e;
        }
        rec[row] = ne;
        rec[16 + row] = row < G ? dsum : 0.f;
    }
    if (blk >= 0 && blk <= tok / kBlock)
        atomicOr(&bitmap[(((int64_t)b * dm.Hkv + h) * nb_cap + blk) * words + (tok >> 5)], 1u << (tok & 31));
}

// ---- re-layout of one 64-token block per workgroup ---------------------------------------------------
// section 0, K rows:  fragment (ks, mt), lane (g, m):  K[64j + 16mt + m][32ks + 8g .. +7]
// section 1, V rows:  the same of V
// section 2, K^T:     fragment (dt, kk), lane (g, m), element e:
//                     K[64j + 32kk + (e<4 ? 4g+e : 16+4g+e-4)][16dt + m]
__global__ __launch_bounds__(256) void pack_bwd_kernel(Dims dm, Tensor k, Tensor v,
                                                        const int32_t *__restrict__ seqlens,
                                                        uint4 *__restrict__ kvb, int32_t nb_cap) {
    __shared__ __align__(16) __bf16 Ks[kBlock * 136];
    __shared__ __align__(16) __bf16 Vs[kBlock * 136];
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = seq_len(dm, seqlens, b);
    if (j * kBlock >= L) return;
    const int tid = threadIdx.x;
    const int sc = tid & 15, sr = tid >> 4;
    const __bf16 *kb = k.ptr + b * k.sb + h * k.sh;
    const __bf16 *vb = v.ptr + b * v.sb + h * v.sh;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = sr + 16 * i, t = j * kBlock + r;
        uint4 xk = {0u, 0u, 0u, 0u}, xv = {0u, 0u, 0u, 0u};
        if (t < L) {
            xk = *reinterpret_cast<const uint4 *>(kb + (int64_t)t * k.st + 8 * sc);
            xv = *reinterpret_cast<const uint4 *>(vb + (int64_t)t * v.st + 8 * sc);
        }
        *reinterpret_cast<uint4 *>(&Ks[r * 136 + 8 * sc]) = xk;
        *reinterpret_cast<uint4 *>(&Vs[r * 136 + 8 * sc]) = xv;
    }
    __syncthreads();
    uint4 *dst = kvb + ((((int64_t)b * dm.Hkv + h) * nb_cap + j) * kBwdBlockU4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;                     // fragment f = c/64, lane = c%64
        const int f = c >> 6, lane = c & 63, m = lane & 15, g = lane >> 4;
        const int ks = f >> 2, mt = f & 3;
        dst[c] = *reinterpret_cast<const uint4 *>(&Ks[(16 * mt + m) * 136 + 32 * ks + 8 * g]);
        dst[1024 + c] = *reinterpret_cast<const uint4 *>(&Vs[(16 * mt + m) * 136 + 32 * ks + 8 * g]);
    }
    const uint16_t *Ku = reinterpret_cast<const uint16_t *>(Ks);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;
        const int f = c >> 6, lane = c & 63, m = lane & 15, g = lane >> 4;
        const int dt = f >> 1, kk = f & 1;
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const int e = 2 * e2;                        // elements e, e+1 are consecutive keys
            const int key = 32 * kk + (e < 4 ? 4 * g + e : 16 + 4 * g + e - 4);
            w[e2] = (uint32_t)Ku[key * 136 + 16 * dt + m] | ((uint32_t)Ku[(key + 1) * 136 + 16 * dt + m] << 16);
        }
        dst[2048 + c] = uint4{w[0], w[1], w[2], w[3]};
    }
}

__device__ inline uint32_t bwd_xcd_contiguous_id(uint32_t bid, uint32_t n) {
    const uint32_t per = n >> 3, rem = n & 7u, x = bid & 7u, slot = bid >> 3;
    return x * per + (x < rem ? x : rem) + slot;
}

// ---- dq: a wavefront owns 2 consecutive tokens of one key-value head ---------------------------------
// A block is processed as two halves of 32 keys; per half six units of 4 fragments (4 KiB each) are
// consumed in this order and rotate through a ring of 4 register buffers (12 units per block):
//   K rows of key tile 2hs, of key tile 2hs+1      -> S^T  = K . Q^T
//   V rows of key tile 2hs, of key tile 2hs+1      -> dP^T = V . dO^T
//   K^T of the half for channel tiles 0..3, 4..7   -> dQ^T += K^T . dS^T
constexpr int kDqTok = 2, kDqRing = 3, kDqUnits = 12;
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(Dims dm, Tensor q, Tensor dout, const uint4 *__restrict__ kvb,
                                                              int32_t nb_cap, const int32_t *__restrict__ seqlens,
                                                              const int32_t *__restrict__ block_idx,
                                                              const float *__restrict__ lse,
                                                              const float *__restrict__ delta, Tensor dq,
                                                              int32_t n_tiles) {
    const uint32_t vid = bwd_xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int tile = vid % n_tiles;
    const int h = (vid / n_tiles) % dm.Hkv;
    const int b = vid / (n_tiles * dm.Hkv);
    const int L = seq_len(dm, seqlens, b);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = (tile * 4 + wave) * kDqTok;            // this wavefront's first token
    if (t0 >= L) return;
    const int b_own = t0 / kBlock;
    const int n = lane & 15, g = lane >> 4;               // MFMA column (query head) and 16-lane group
    const int G = dm.G;
    const float c = dm.scale_log2;

    bf16x8 qf[kDqTok][4], gf[kDqTok][4];
    f32x4 acc[kDqTok][8];
    float neg_lse2[kDqTok], dlt[kDqTok];                  // per lane: its head's -lse*log2(e) and D
    int own[kDqTok];
#pragma unroll
    for (int u = 0; u < kDqTok; ++u) {
        const int tok = t0 + u;
        const bool live = tok < L && n < G;
        const int64_t row = (int64_t)(h * G + min(n, G - 1));
        const int tk = min(tok, L - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[u][ks] = load8(q.ptr + b * q.sb + (int64_t)tk * q.st + row * q.sh + 32 * ks + 8 * g);
            gf[u][ks] = load8(dout.ptr + b * dout.sb + (int64_t)tk * dout.st + row * dout.sh + 32 * ks + 8 * g);
        }
        const float ls = lse[((int64_t)b * dm.max_seqlen + tk) * dm.Hq + row];
        dlt[u] = delta[((int64_t)b * dm.max_seqlen + tk) * dm.Hq + row];
        // p = 2^(s*c - lse*log2e); a dead column (no such token or head, or a row that attended nothing) gets p = 0
        neg_lse2[u] = (live && ls > -INFINITY) ? -ls * kLog2e : -INFINITY;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) acc[u][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        int e = kBwdNone;
        if (tok < L && lane < dm.topk) {
            const int x = block_idx[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * dm.topk + lane];
            if (x >= 0 && x <= b_own) e = x;
        }
        own[u] = e;
    }
    // ascending union of the two block lists by counting (an entry's place = number of distinct smaller entries)
    // (a block listed twice in one row, against the contract, counts once: the copy in the higher lane is dropped)
    int w[kDqTok];
#pragma unroll
    for (int u = 0; u < kDqTok; ++u) {
        bool dup = false;
        for (int j = 0; j < dm.topk; ++j) dup |= j < lane && __builtin_amdgcn_readlane(own[u], j) == own[u];
        if (u == 1)
            for (int j = 0; j < dm.topk; ++j) dup |= __builtin_amdgcn_readlane(own[0], j) == own[1];
        w[u] = dup ? kBwdNone : own[u];
    }
    int rank[kDqTok] = {0, 0}, bits[kDqTok] = {0, 0};
#pragma unroll
    for (int u2 = 0; u2 < kDqTok; ++u2)
        for (int j = 0; j < dm.topk; ++j) {
            const int wj = __builtin_amdgcn_readlane(w[u2], j), xj = __builtin_amdgcn_readlane(own[u2], j);
#pragma unroll
            for (int u = 0; u < kDqTok; ++u) {
                rank[u] += wj < w[u] ? 1 : 0;
                bits[u] |= xj == w[u] ? 1 << u2 : 0;
            }
        }
    __shared__ int ulist[4][64 * kDqTok];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < kDqTok; ++u) {
        const bool have = w[u] != kBwdNone;
        if (have) ulist[wave][rank[u]] = w[u] | (bits[u] << kBwdBlkBits);
        cnt += __popcll(__ballot(have));
    }
    int ul[kDqTok];
#pragma unroll
    for (int r = 0; r < kDqTok; ++r) ul[r] = ulist[wave][64 * r + lane];
    auto union_entry = [&](int i) __attribute__((always_inline)) {
        int e = __builtin_amdgcn_readlane(ul[0], i & 63);
        if ((i >> 6) == 1) e = __builtin_amdgcn_readlane(ul[1], i & 63);
        return e;
    };

    const u32x4 *kv_lane = reinterpret_cast<const u32x4 *>(kvb) + ((int64_t)b * dm.Hkv + h) * nb_cap * kBwdBlockU4 + lane;
    u32x4 ring[kDqRing][4];
    auto issue = [&](int unit, const u32x4 *bp) __attribute__((always_inline)) {
        const int hs = unit / 6, r = unit % 6;
        if (r < 4) {                                      // K rows (section 0) or V rows (section 1), key tile 2hs + r%2
            const int sec = r >> 1, mt = 2 * hs + (r & 1);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) ring[unit % kDqRing][ks] = bp[(sec * 16 + ks * 4 + mt) * 64];
        } else {                                          // K^T (section 2), channel tiles 4(r-4) .. +3 of half hs
#pragma unroll
            for (int i = 0; i < 4; ++i) ring[unit % kDqRing][i] = bp[(32 + (4 * (r - 4) + i) * 2 + hs) * 64];
        }
    };

    __builtin_amdgcn_s_waitcnt(0);                        // nothing of the prologue may still be pending inside the ring loop
    if (cnt > 0) {
        const u32x4 *bp = kv_lane + (int64_t)(union_entry(0) & kBwdBlkMask) * kBwdBlockU4;
#pragma unroll
        for (int unit = 0; unit < kDqRing; ++unit) issue(unit, bp);
    }
    for (int ci = 0; ci < cnt; ++ci) {
        const int e = union_entry(ci);
        const int blk = e & kBwdBlkMask, mem = e >> kBwdBlkBits;
        const int en = union_entry(ci + 1 < cnt ? ci + 1 : ci);
        const u32x4 *bp = kv_lane + (int64_t)blk * kBwdBlockU4;
        const u32x4 *bn = kv_lane + (int64_t)(en & kBwdBlkMask) * kBwdBlockU4;
        const int key0 = blk * kBlock;
        const bool edge = blk == b_own;
        auto refill = [&](int unit) __attribute__((always_inline)) {
            if (unit + kDqRing < kDqUnits) issue(unit + kDqRing, bp);
            else issue(unit + kDqRing - kDqUnits, bn);    // (a harmless re-read of this block at the tail)
        };
#pragma unroll
        for (int hs = 0; hs < 2; ++hs) {
            f32x4 s[kDqTok][2], dp[kDqTok][2];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int unit = 6 * hs + r;
#pragma unroll
                for (int u = 0; u < kDqTok; ++u) {
                    if (!((mem >> u) & 1)) continue;
                    f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        a = mfma16(__builtin_bit_cast(bf16x8, ring[unit % kDqRing][ks]), r < 2 ? qf[u][ks] : gf[u][ks], a);
                    if (r < 2) s[u][r] = a;
                    else dp[u][r - 2] = a;
                }
                refill(unit);
            }
            bf16x8 dsf[kDqTok];
#pragma unroll
            for (int u = 0; u < kDqTok; ++u) {
                if (!((mem >> u) & 1)) continue;
                const int tok = t0 + u;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float p = fast_exp2(__builtin_fmaf(s[u][t][j], c, neg_lse2[u]));
                        if (edge && key0 + 32 * hs + 16 * t + 4 * g + j > tok) p = 0.f;
                        dsf[u][4 * t + j] = (__bf16)(p * (dp[u][t][j] - dlt[u]));
                    }
            }
#pragma unroll
            for (int r = 4; r < 6; ++r) {
                const int unit = 6 * hs + r;
#pragma unroll
                for (int u = 0; u < kDqTok; ++u) {
                    if (!((mem >> u) & 1)) continue;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[u][4 * (r - 4) + i] =
                            mfma16(__builtin_bit_cast(bf16x8, ring[unit % kDqRing][i]), dsf[u], acc[u][4 * (r - 4) + i]);
                }
                refill(unit);
            }
        }
    }
    // ---- write: lane holds channels 16*dt + 4*g .. +3 of head n ------------------------------------------
    const float scale = c * kLn2;
#pragma unroll
    for (int u = 0; u < kDqTok; ++u) {
        const int tok = t0 + u;
        if (tok >= L || n >= G) continue;
        __bf16 *op = dq.ptr + b * dq.sb + (int64_t)tok * dq.st + (int64_t)(h * G + n) * dq.sh + 4 * g;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            bf16x4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = (__bf16)(acc[u][dt][j] * scale);
            *reinterpret_cast<uint2 *>(op + 16 * dt) = __builtin_bit_cast(uint2, r);
        }
    }
}

// ---- dk, dv of one block from the tokens that selected it ------------------------------------------------------
// 256 threads: a workgroup handles member tokens of block j that lie in one segment of the sequence (all of
// them, or one slice of the list when there are many).  The member tokens are compacted from the bitmap into a
// list and walked in pairs; rows = (token of the pair, head).  Every pair has two phases with a barrier between:
//   phase 1, wave = (token u, key half kh), 16x16x32 MFMAs: S = Q.K^T and dP = dO.V^T for the token's 16 heads
//            and the half's 32 keys (A = the token's q / dout rows from LDS, B = K / V rows of the keys, held
//            in registers), then P = exp(S - lse) and dS = P (dP - D), left in LDS as bf16 in the layout of a
//            32x32x16 B operand (lane = key, 8 heads of one token per lane);
//   phase 2, wave = channel quarter cq, 32x32x16 MFMAs: dV^T[c, key] += dO^T[c, row] . P[row, key] and
//            dK^T[c, key] += Q^T[c, row] . dS[row, key] for channels 32cq .. +31 and all 64 keys: A = the same
//            staged rows read through the transposing LDS load (each fragment feeds both key halves), B = P / dS.
// Nothing is computed twice, and a wavefront keeps 64 accumulator registers next to the 64 of its K and V operands.
// Staging: the 16 KiB of q and dout rows of a pair (and its 64 scalars) go from memory straight into LDS (no
// registers, no vector instructions) two pairs ahead; three slots rotate.  The slots are three objects and the
// loop is unrolled by three, so that the compiler's wait counts let reads of one slot run under the copies into
// another.  A row is 256 bytes; its sixteen 16-byte pieces are stored XOR-swizzled with the head's two bit
// pairs exchanged: an operand load of phase 1 takes one piece from each of 16 rows, a transposing load 32 bytes
// from each of 4 consecutive rows, and both then touch every bank once.
constexpr int kBwdSlices = 4;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
struct __align__(16) BwdSlot {
    uint16_t rows[2][32][kHeadDim];                       // [q | dout][(token, head)][channel]: 16 KiB
    float ld[64];                                         // [exponent offset of token a, of b | D of token a, of b][head]
};
struct __align__(16) BwdExchange {
    uint4 frag[2][2][2][2][64];                           // [buffer][P | dS][token][key half][lane = (key, head group)]: 16 KiB
};
__device__ __forceinline__ int bwd_swizzle(int head) { return ((head & 3) << 2) | ((head >> 2) & 3); }
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// 4 rows x 16 channels per 16-lane group, transposed: lane i of the group gets channel i of the four rows its
// group addressed (source lane s: row s/4, channels 4(s%4) .. +3)
__device__ __forceinline__ s16x4 lds_read_tr16(const char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
}

template <int kSegTokens>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkdv_kernel(Dims dm, Tensor q, Tensor dout, const uint4 *__restrict__ kvb,
                                                                int32_t nb_cap, const int32_t *__restrict__ seqlens,
                                                                const float *__restrict__ rowc,
                                                                const uint32_t *__restrict__ bitmap, int32_t words,
                                                                float *__restrict__ acc_dk, float *__restrict__ acc_dv) {
    constexpr int kSegWords = kSegTokens / 32;
    constexpr int kSegWordsPerLane = kSegWords / 64;      // the member list is compacted by one wavefront
    static_assert(kSegWords % 64 == 0 && kSegTokens <= 65536, "whole words per lane; 16-bit offsets in the member list");
    __shared__ uint16_t list[kSegTokens / kBwdSlices];   // this workgroup's member tokens as offsets into the segment
    __shared__ BwdSlot slot0, slot1, slot2;
    __shared__ BwdExchange ex;
    __shared__ int total_s;
    // grid (blocks, segments x slices, B*Hkv): workgroups that run at the same time work on neighbouring blocks
    // of one segment and find its tokens' rows in the caches; a (block, segment) unit with many members is
    // shared by up to kBwdSlices workgroups, each taking kSliceTokens consecutive members
    constexpr int kSliceTokens = kSegTokens / kBwdSlices;
    const int j = blockIdx.x, seg = blockIdx.y / kBwdSlices, slice = blockIdx.y - seg * kBwdSlices;
    const int b = blockIdx.z / dm.Hkv, h = blockIdx.z - b * dm.Hkv;
    const int L = seq_len(dm, seqlens, b);
    if ((seg + 1) * kSegTokens <= j * kBlock || seg * kSegTokens >= L || j * kBlock >= L) return;   // no member can be here
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = dm.G;
    const float c = dm.scale_log2;
    const int64_t bh = (int64_t)b * dm.Hkv + h;
    // ---- member tokens of this segment, ascending (wave 0) ----------------------------------------------
    uint32_t word[kSegWordsPerLane];                      // consecutive words per lane: the list comes out ascending
    int before = 0, mine = 0;
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < kSegWordsPerLane; ++i) {
            word[i] = bitmap[(bh * nb_cap + j) * words + seg * kSegWords + lane * kSegWordsPerLane + i];
            mine += __popc(word[i]);
        }
        before = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int x = __shfl_up(before, o);
            if (lane >= o) before += x;
        }
        if (lane == 63) total_s = before;
        before -= mine;
    }
    __syncthreads();
    const int first = slice * kSliceTokens;               // this workgroup's members: first .. first + total - 1 of the unit
    const int total = min(total_s - first, kSliceTokens);
    if (total <= 0) return;                               // uniform
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < kSegWordsPerLane; ++i) {
            uint32_t w = word[i];
            while (w) {
                const int bit = __ffs(w) - 1;
                w &= w - 1;
                const int at = before++ - first;
                if (at >= 0 && at < kSliceTokens) list[at] = (uint16_t)((lane * kSegWordsPerLane + i) * 32 + bit);
            }
        }
    }
    __syncthreads();
    const int n_pairs = (total + 1) >> 1;
    const int n = lane & 15, g = lane >> 4;               // 16x16x32 roles: row / column, k group
    const int c32 = lane & 31, hf = lane >> 5;            // 32x32x16 roles
    const int u = wave >> 1, kh = wave & 1;               // phase 1: token of the pair, key half
    const int cq = wave;                                  // phase 2: channel quarter
    // ---- phase 1 B operands: K and V rows of keys 32kh + 16t + n, channels 32ks + 8g .. +7 ---------------------
    const u32x4 *blk = reinterpret_cast<const u32x4 *>(kvb) + (bh * nb_cap + j) * kBwdBlockU4 + lane;
    bf16x8 kB[2][4], vB[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            kB[t][ks] = __builtin_bit_cast(bf16x8, blk[(ks * 4 + 2 * kh + t) * 64]);
            vB[t][ks] = __builtin_bit_cast(bf16x8, blk[(16 + ks * 4 + 2 * kh + t) * 64]);
        }
    f32x16 dkT[2], dvT[2];                                // [key half]: channels 32cq .. +31 x 32 keys
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) dkT[i][v] = dvT[i][v] = 0.f;

    // staging: wave w copies one token's 16 rows of one tensor (token w&1 of the pair, q for w < 2, dout else): four
    // 1 KiB copies of four heads each, all from one token offset; lane = (head 4i + lane/16, piece lane%16 of the
    // LDS row = piece (lane%16) ^ swizzle(head) of the row in memory)
    const Tensor &s_t = wave < 2 ? q : dout;
    const __bf16 *s_base = s_t.ptr + b * s_t.sb + (int64_t)(h * G) * s_t.sh;
    int32_t s_off[4];                                     // elements from the token's first head of the group
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int head = 4 * i + (lane >> 4);
        s_off[i] = (int32_t)(min(head, G - 1) * s_t.sh) + 8 * ((lane & 15) ^ bwd_swizzle(head));
    }
    const float *s_f = rowc + ((int64_t)b * dm.max_seqlen * dm.Hkv + h) * 32 + 16 * (lane >> 5) + (lane & 15);   // + 32 Hkv tok
    auto stage = [&](BwdSlot &dst, int p) __attribute__((always_inline)) {
        const int tok = seg * kSegTokens + list[min(2 * p + (wave & 1), total - 1)];
        const __bf16 *src = s_base + (int64_t)tok * s_t.st;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + s_off[i]),
                                             (__attribute__((address_space(3))) void *)&dst.rows[wave >> 1][16 * (wave & 1) + 4 * i][0],
                                             16, 0, 0);
        if (wave == 0) {
            const int tb = seg * kSegTokens + list[min(2 * p + 1, total - 1)];
            const int tk = ((lane >> 4) & 1) ? tb : tok;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(s_f + (int64_t)tk * dm.Hkv * 32),
                                             (__attribute__((address_space(3))) void *)&dst.ld[0], 4, 0, 0);
        }
    };
    // LDS addresses of the operand loads, the parts that depend on the lane
    const uint32_t a_row = (uint32_t)(16 * u + n) * 256u + (uint32_t)((g ^ bwd_swizzle(n)) << 4);   // piece 4ks + g of the row: ^ (ks << 6)
    const uint32_t t_r = 4u * hf + ((lane & 15) >> 2), t_c = 2u * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    // (channel quarter cq starts at piece 4cq; rows 8rd + t_r have swizzle 2rd ^ swizzle(t_r))
    const uint32_t a_tr = t_r * 256u + ((t_c ^ (uint32_t)bwd_swizzle((int)t_r) ^ (4u * cq)) << 4) + 8u * (lane & 1);   // ^ (2rd << 4), + (16 s2 + 8 rd) rows
    // where this lane's four probabilities of a key go in the exchange: consumer lane (key 16t + n, head group g & 1),
    // elements 4 (g >> 1) .. +3
    const uint32_t x_put = (uint32_t)((n + 32 * (g & 1)) * 16 + 8 * (g >> 1));   // + 256 t bytes

    auto phase1 = [&](const BwdSlot &cur, int p) __attribute__((always_inline)) {
        const int tk = seg * kSegTokens + list[min(2 * p + u, total - 1)];
        const bool valid = 2 * p + u < total;
        const char *xq = reinterpret_cast<const char *>(&cur.rows[0][0][0]);
        const char *xg = reinterpret_cast<const char *>(&cur.rows[1][0][0]);
        f32x4 sacc[2], dp[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) sacc[t] = dp[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 qa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(xq + (a_row ^ (uint32_t)(ks << 6))));
            const bf16x8 ga = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(xg + (a_row ^ (uint32_t)(ks << 6))));
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                sacc[t] = mfma16(qa, kB[t][ks], sacc[t]);
                dp[t] = mfma16(ga, vB[t][ks], dp[t]);
            }
        }
        // accumulator entry r of tile t: head 4g + r (row), key 32kh + 16t + n (column)
        const float4 n4 = *reinterpret_cast<const float4 *>(&cur.ld[16 * u + 4 * g]);
        const float4 d4 = *reinterpret_cast<const float4 *>(&cur.ld[32 + 16 * u + 4 * g]);
        const float nl[4] = {n4.x, n4.y, n4.z, n4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
        char *xp = reinterpret_cast<char *>(&ex.frag[p & 1][0][u][kh][0]) + x_put;
        char *xs = reinterpret_cast<char *>(&ex.frag[p & 1][1][u][kh][0]) + x_put;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            // padding of the list and the causal edge inside the own block: the exponent's offset becomes -inf
            const float bias = (!valid | (j * kBlock + 32 * kh + 16 * t + n > tk)) ? -INFINITY : 0.f;
            bf16x4 pb, sb;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float pr = fast_exp2(__builtin_fmaf(sacc[t][r], c, nl[r] + bias));
                pb[r] = (__bf16)pr;
                sb[r] = (__bf16)(pr * (dp[t][r] - dl[r]));
            }
            *reinterpret_cast<uint2 *>(xp + 256 * t) = __builtin_bit_cast(uint2, pb);
            *reinterpret_cast<uint2 *>(xs + 256 * t) = __builtin_bit_cast(uint2, sb);
        }
    };
    auto phase2 = [&](const BwdSlot &cur, int p) __attribute__((always_inline)) {
        const char *xq = reinterpret_cast<const char *>(&cur.rows[0][0][0]);
        const char *xg = reinterpret_cast<const char *>(&cur.rows[1][0][0]);
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const uint32_t o0 = a_tr + (uint32_t)(16 * s2) * 256u;
            const uint32_t o1 = (a_tr ^ (uint32_t)(2 << 4)) + (uint32_t)(16 * s2 + 8) * 256u;
            const s16x4 g0 = lds_read_tr16(xg + o0), g1 = lds_read_tr16(xg + o1);
            const s16x4 q0 = lds_read_tr16(xq + o0), q1 = lds_read_tr16(xq + o1);
            const bf16x8 ag = __builtin_bit_cast(bf16x8, __builtin_shufflevector(g0, g1, 0, 1, 2, 3, 4, 5, 6, 7));
            const bf16x8 aq = __builtin_bit_cast(bf16x8, __builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2) {
                const bf16x8 pf = __builtin_bit_cast(bf16x8, ex.frag[p & 1][0][s2][k2][lane]);
                const bf16x8 sf = __builtin_bit_cast(bf16x8, ex.frag[p & 1][1][s2][k2][lane]);
                dvT[k2] = mfma32(ag, pf, dvT[k2]);
                dkT[k2] = mfma32(aq, sf, dkT[k2]);
            }
        }
    };
    // pair p: phase 1, barrier, phase 2; the copies for pair p + 2 go out right after the barrier, into the slot
    // whose last reads (phase 2 of pair p - 1) everyone has finished by then, and have a whole pair's time to land.
    // The trip count is rounded up to a multiple of three and nothing in the loop is conditional (pairs past the
    // end are copies of the last token with every probability zero): at a join of two paths the compiler would
    // wait for every copy in flight.
    auto pair_step = [&](const BwdSlot &cur, BwdSlot &third, int p) __attribute__((always_inline)) {
        phase1(cur, p);
        __builtin_amdgcn_s_waitcnt(0);                    // this wavefront's copies for pair p + 1 have landed
        __syncthreads();                                  // everyone's have; P and dS of pair p are in place
        stage(third, p + 2);
        phase2(cur, p);
    };
    stage(slot0, 0);
    stage(slot1, 1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int p = 0; p < n_pairs; p += 3) {
        pair_step(slot0, slot2, p);
        pair_step(slot1, slot0, p + 1);
        pair_step(slot2, slot1, p + 2);
    }
    __builtin_amdgcn_s_waitcnt(0);                        // the last copies (never used) have landed: the slots are reused below
    // ---- merge: a lane holds channels 32cq + 8(v/4) + 4hf + v%4 of key 32kh' + c32.  The tiles are turned through
    // LDS (the staging slots, 8 KiB per wavefront) so that one atomic instruction covers the 32 channels of two
    // keys: two cache lines instead of 64. --------------------------------------------------------------------
    __syncthreads();                                      // every wavefront is past its last read of the staging slots
    float *tile = reinterpret_cast<float *>(wave < 2 ? &slot0.rows[0][0][0] : &slot1.rows[0][0][0]) + (wave & 1) * 2048;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        // [key 0 .. 63][16-byte piece ^ (key & 7)][4 channels]
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const f32x16 &t = which ? dvT[k2] : dkT[k2];
                const int key = 32 * k2 + c32, piece = 2 * v4 + hf;   // channels 4 piece .. +3 of the wave's 32
                *reinterpret_cast<float4 *>(tile + key * 32 + ((piece ^ (key & 7)) << 2)) =
                    float4{t[4 * v4], t[4 * v4 + 1], t[4 * v4 + 2], t[4 * v4 + 3]};
            }
        // (same wavefront wrote and reads: LDS keeps the order)
        float *acc = (which ? acc_dv : acc_dk) + (bh * dm.max_seqlen + (int64_t)j * kBlock + hf) * kHeadDim + 32 * cq + c32;
#pragma unroll 8
        for (int i = 0; i < 32; ++i) {
            const int key = 2 * i + hf;
            const float x = tile[key * 32 + ((((c32 >> 2) ^ (key & 7)) << 2) | (c32 & 3))];
            if (j * kBlock + key < L) unsafeAtomicAdd(acc + (int64_t)(2 * i) * kHeadDim, x);
        }
    }
}

// ---- fp32 accumulators -> bf16 gradients ------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_finish_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                          const float *__restrict__ acc_dk,
                                                          const float *__restrict__ acc_dv, Tensor dk, Tensor dv) {
    const int b = blockIdx.z, h = blockIdx.y;
    const int L = seq_len(dm, seqlens, b);
    const int t = blockIdx.x * 16 + (threadIdx.x >> 4), c8 = (threadIdx.x & 15) * 8;
    if (t >= L) return;
    const float scale = dm.scale_log2 * kLn2;
    const int64_t src = (((int64_t)b * dm.Hkv + h) * dm.max_seqlen + t) * kHeadDim + c8;
    const float4 k0 = *reinterpret_cast<const float4 *>(acc_dk + src), k1 = *reinterpret_cast<const float4 *>(acc_dk + src + 4);
    const float4 v0 = *reinterpret_cast<const float4 *>(acc_dv + src), v1 = *reinterpret_cast<const float4 *>(acc_dv + src + 4);
    const float kf[8] = {k0.x, k0.y, k0.z, k0.w, k1.x, k1.y, k1.z, k1.w};
    const float vf[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    bf16x8 ko, vo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        ko[e] = (__bf16)(kf[e] * scale);
        vo[e] = (__bf16)vf[e];
    }
    *reinterpret_cast<uint4 *>(dk.ptr + b * dk.sb + h * dk.sh + (int64_t)t * dk.st + c8) = __builtin_bit_cast(uint4, ko);
    *reinterpret_cast<uint4 *>(dv.ptr + b * dv.sb + h * dv.sh + (int64_t)t * dv.st + c8) = __builtin_bit_cast(uint4, vo);
}

int launch_attn_bwd(const Dims &dm, Tensor q, Tensor k, Tensor v, Tensor out, Tensor dout, const float *lse,
                    const int32_t *seqlens, const int32_t *block_idx, Tensor dq, Tensor dk, Tensor dv, void *ws,
                    hipStream_t stream) {
    if (dm.batch <= 0 || dm.max_seqlen <= 0) return 0;
    const BwdLayout l = bwd_layout(dm);
    char *base = reinterpret_cast<char *>(ws);
    uint4 *kvb = reinterpret_cast<uint4 *>(base + l.kvb);
    float *delta = reinterpret_cast<float *>(base + l.delta);
    float *rowc = reinterpret_cast<float *>(base + l.rowc);
    uint32_t *bitmap = reinterpret_cast<uint32_t *>(base + l.bitmap);
    float *acc_dk = reinterpret_cast<float *>(base + l.acc_dk), *acc_dv = reinterpret_cast<float *>(base + l.acc_dv);
    const int T = dm.max_seqlen;
    timing_begin("bwd_zero_kernel", stream);
    hipLaunchKernelGGL(bwd_zero_kernel, dim3(2048), dim3(256), 0, stream, reinterpret_cast<uint4 *>(base + l.zero_begin),
                       l.zero_bytes / sizeof(uint4));
    timing_end(stream);
    timing_begin("bwd_prep_kernel", stream);
    hipLaunchKernelGGL(bwd_prep_kernel, dim3((T + 3) / 4, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, out, dout,
                       seqlens, block_idx, lse, delta, rowc, bitmap, l.nb_cap, l.words);
    timing_end(stream);
    timing_begin("pack_bwd_kernel", stream);
    hipLaunchKernelGGL(pack_bwd_kernel, dim3(l.nb_cap, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, k, v, seqlens, kvb,
                       l.nb_cap);
    timing_end(stream);
    const int32_t n_tiles = (T + 4 * kDqTok - 1) / (4 * kDqTok);
    timing_begin("attn_bwd_dq_kernel", stream);
    hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3((uint32_t)((int64_t)n_tiles * dm.Hkv * dm.batch)), dim3(256), 0, stream,
                       dm, q, dout, kvb, l.nb_cap, seqlens, block_idx, lse, delta, dq, n_tiles);
    timing_end(stream);
    timing_begin("attn_bwd_dkdv_kernel", stream);
    if (bwd_seg_tokens(dm) == 8192)
        hipLaunchKernelGGL(attn_bwd_dkdv_kernel<8192>, dim3(l.nb_cap, l.words / 256 * kBwdSlices, dm.batch * dm.Hkv), dim3(256), 0,
                           stream, dm, q, dout, kvb, l.nb_cap, seqlens, rowc, bitmap, l.words, acc_dk, acc_dv);
    else
        hipLaunchKernelGGL(attn_bwd_dkdv_kernel<2048>, dim3(l.nb_cap, l.words / 64 * kBwdSlices, dm.batch * dm.Hkv), dim3(256), 0,
                           stream, dm, q, dout, kvb, l.nb_cap, seqlens, rowc, bitmap, l.words, acc_dk, acc_dv);
    timing_end(stream);
    timing_begin("bwd_finish_kernel", stream);
    hipLaunchKernelGGL(bwd_finish_kernel, dim3((T + 15) / 16, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, seqlens,
                       acc_dk, acc_dv, dk, dv);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
