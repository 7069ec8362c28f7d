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
//   bwd_prep_kernel     D and the membership bits of every token
//   pack_bwd_kernel     fragment-major copies of every block: K rows, V rows, K transposed
//   attn_bwd_dq_kernel  wavefront = 2 tokens, walks the union of their block lists:
//                       S^T = K.Q^T, dP^T = V.dO^T, dQ^T += K^T.dS^T
//   attn_bwd_dkdv_kernel  wavefront = 16 keys of a block, walks the member tokens of one
//                       2048-token segment in pairs: S = Q.K^T, dP = dO.V^T,
//                       dV^T += dO^T.P, dK^T += Q^T.dS; fp32 atomics merge the segments
//   bwd_finish_kernel   fp32 accumulators -> bf16 dk (times scale), dv
// As in the forward, every second contraction takes its B operand straight from the accumulator
// layout of the first (lane = column, 4 consecutive rows per 16-lane group), with the contraction
// index of the A fragments permuted to match.
#include "common.h"

namespace infllmv2 {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBwdBlockU4 = 3 * 16 * 64;              // uint4 per packed block: K rows, V rows, K^T (48 KiB)
// Member tokens of one dk/dv workgroup come from one segment of the sequence.  Short segments give
// more workgroups (better balance at 32K tokens), long ones fewer prologues and merges per block
// (at 128K tokens most (block, segment) units hold a handful of members).
static inline int bwd_seg_tokens(const Dims &dm) { return dm.max_seqlen > 65536 ? 4096 : 2048; }
constexpr int kBwdNone = 0x7fffffff;
constexpr int kBwdBlkBits = 27, kBwdBlkMask = (1 << kBwdBlkBits) - 1;

struct BwdLayout {
    int32_t nb_cap, words;                            // blocks per sequence; bitmap words per block row (multiple of 64)
    size_t kvb, delta, bitmap, acc_dk, acc_dv, total; // byte offsets into the workspace
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
                                                        float *__restrict__ delta, uint32_t *__restrict__ bitmap,
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

// ---- dk, dv: a wavefront owns 16 keys of a block ---------------------------------------------------------
// grid (nb_cap, n_seg, B*Hkv), 256 threads: workgroup (j, seg) handles the member tokens of block j
// that lie in tokens [2048 seg, 2048 seg + 2047]; wave w the keys 64j + 16w .. +15.  The member
// tokens are compacted from the bitmap into a list and walked two at a time.  All four waves need
// the same 16 KiB of q and dout rows per pair, so the workgroup fetches each pair once: every
// thread keeps its 1/256 of the next three pairs in registers (memory latency is several times the
// arithmetic of a pair) and drops a pair into one of two LDS buffers one step before it is used,
// as rows and, transposed in registers, as columns.
//   S  [head, key] = Q[tok] . K^T        A = q rows of the token (lane = head), B = K rows (registers)
//   dP [head, key] = dO[tok] . V^T
//   dV^T[c, key]  += dO^T[c, (tok, head)] . P[(tok, head), key]      A = the staged columns,
//   dK^T[c, key]  += Q^T [c, (tok, head)] . dS[(tok, head), key]     B = P / dS
// as they sit in the accumulators of the first two products.
constexpr int kRowPitch = kHeadDim + 8;               // bf16 per staged row (272 bytes: rows start 4 banks apart)
constexpr int kPairRows = 2 * 2 * 16;                 // q rows of two tokens, dout rows of two tokens
constexpr int kDepth = 3;                             // pairs in flight per thread
template <int kSegTokens>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkdv_kernel(Dims dm, Tensor q, Tensor dout, const uint4 *__restrict__ kvb,
                                                                int32_t nb_cap, const int32_t *__restrict__ seqlens,
                                                                const float *__restrict__ lse,
                                                                const float *__restrict__ delta,
                                                                const uint32_t *__restrict__ bitmap, int32_t words,
                                                                float *__restrict__ acc_dk, float *__restrict__ acc_dv) {
    constexpr int kSegWords = kSegTokens / 32;
    constexpr int kSegWordsPerLane = kSegWords / 64;      // the member list is compacted by one wavefront
    static_assert(kSegWords % 64 == 0 && kSegTokens <= 65536, "whole words per lane; 16-bit offsets in the member list");
    __shared__ uint16_t list[kSegTokens];                // member tokens as offsets into the segment
    __shared__ __align__(16) uint16_t stage[2][kPairRows * kRowPitch];   // [buffer][(q | dout, token, head)][channel]
    __shared__ __align__(16) uint16_t stageT[2][2 * 8 * 64 * 8];         // [buffer][(q | dout, dt, lane)][token][4 heads]
    __shared__ __align__(16) float ld[2][2][2][16];       // [buffer][lse | D][token of the pair][head]
    __shared__ int total_s;
    const int j = blockIdx.x, seg = blockIdx.y;
    const int b = blockIdx.z / dm.Hkv, h = blockIdx.z - b * dm.Hkv;
    const int L = seq_len(dm, seqlens, b);
    if ((seg + 1) * kSegTokens <= j * kBlock || seg * kSegTokens >= L || j * kBlock >= L) return;   // no member can be here
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int G = dm.G;
    const float c = dm.scale_log2;
    const int64_t bh = (int64_t)b * dm.Hkv + h;
    // ---- member tokens of this segment, ascending (wave 0) ----------------------------------------------
    if (wave == 0) {
        uint32_t word[kSegWordsPerLane];                  // consecutive words per lane: the list comes out ascending
        int mine = 0;
#pragma unroll
        for (int i = 0; i < kSegWordsPerLane; ++i) {
            word[i] = bitmap[(bh * nb_cap + j) * words + seg * kSegWords + lane * kSegWordsPerLane + i];
            mine += __popc(word[i]);
        }
        int before = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int x = __shfl_up(before, o);
            if (lane >= o) before += x;
        }
        if (lane == 63) total_s = before;
        before -= mine;
#pragma unroll
        for (int i = 0; i < kSegWordsPerLane; ++i) {
            uint32_t w = word[i];
            while (w) {
                const int bit = __ffs(w) - 1;
                w &= w - 1;
                list[before++] = (uint16_t)((lane * kSegWordsPerLane + i) * 32 + bit);
            }
        }
    }
    __syncthreads();
    const int total = total_s;
    if (total == 0) return;                               // uniform
    const int n_pairs = (total + 1) >> 1;
    // ---- this wave's keys as B operands: lane (n, g) = key 16w + n, channels 32ks + 8g .. +7 -----------
    const u32x4 *blk_lane = reinterpret_cast<const u32x4 *>(kvb) + (bh * nb_cap + j) * kBwdBlockU4 + lane;
    bf16x8 kB[4], vB[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        kB[ks] = __builtin_bit_cast(bf16x8, blk_lane[(ks * 4 + wave) * 64]);
        vB[ks] = __builtin_bit_cast(bf16x8, blk_lane[(16 + ks * 4 + wave) * 64]);
    }
    f32x4 dkT[8], dvT[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) dkT[dt] = dvT[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int key = j * kBlock + 16 * wave + n;           // this lane's key (column of S)

    // this thread's share of a pair: a 4-head x 8-channel patch of one of the four 16-row tiles
    // (tile = tid>>6: q of token a, q of token b, dout of token a, dout of token b; heads 4*f_g .. +3,
    // channels 8*f_pc .. +7), one scalar.  The patch goes to LDS twice: as rows (A operands of the
    // first products, 16 bytes per head) and transposed (A operands of the second products: lane
    // (n = channel, g) reads heads 4g .. 4g+3 of its channel as 8 bytes).
    const int f_tile = tid >> 6, f_g = (tid >> 4) & 3, f_pc = tid & 15;
    const Tensor &src = (f_tile & 2) ? dout : q;
    const __bf16 *f_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        f_base[e] = src.ptr + b * src.sb + (int64_t)(h * G + min(4 * f_g + e, G - 1)) * src.sh + 8 * f_pc;
    u32x4 r[kDepth][4];                                   // (ext vectors: arrays of HIP's uint4 struct end up in scratch)
    float rf[kDepth];
    auto fetch = [&](int p, int st) __attribute__((always_inline)) {
        const int ta = seg * kSegTokens + list[min(2 * p, total - 1)], tb = seg * kSegTokens + list[min(2 * p + 1, total - 1)];
        const int tok = (f_tile & 1) ? tb : ta;
#pragma unroll
        for (int e = 0; e < 4; ++e) r[st][e] = *reinterpret_cast<const u32x4 *>(f_base[e] + (int64_t)tok * src.st);
        {   // every thread loads (a fixed number of loads per step keeps the wait counts exact); 64 values are kept
            const int t2 = ((tid >> 4) & 1) ? tb : ta;
            const int64_t o = ((int64_t)b * dm.max_seqlen + t2) * dm.Hq + h * G + min(tid & 15, G - 1);
            rf[st] = ((tid >> 5) & 1 ? delta : lse)[o];
        }
    };
    auto stash = [&](int buf, int st) __attribute__((always_inline)) {
        uint16_t *dst = &stage[buf][(f_tile * 16 + 4 * f_g) * kRowPitch + 8 * f_pc];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            u32x4 x = r[st][e];
            if (4 * f_g + e >= G) x = u32x4{0u, 0u, 0u, 0u};        // heads past the group are zero rows
            *reinterpret_cast<u32x4 *>(dst + e * kRowPitch) = x;
        }
        // transposed: channel 8*f_pc + cc -> fragment dt = f_pc/2, lane (f_g, m = 8*(f_pc&1) + cc): heads 4f_g .. +3.
        // Layout [q | dout][dt][lane][token of the pair][4 heads]: a lane finds the 16 bytes of one A operand
        // in one piece.  The 16-byte slots of a fragment are XOR-swizzled with dt & 7 so that the 16 lanes of
        // a store, which differ in dt, spread over all banks; a load has dt fixed and stays a permutation.
        const int t_dt = f_pc >> 1;
        u32x2 *trow = reinterpret_cast<u32x2 *>(&stageT[buf][(((f_tile >> 1) * 8 + t_dt) * 64) * 8]) + (f_tile & 1);
        const int t_lane = f_g * 16 + 8 * (f_pc & 1);
#pragma unroll
        for (int c2 = 0; c2 < 4; ++c2) {                  // channels 2*c2, 2*c2+1 sit in word c2 of every head's piece
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (4 * f_g + e < G) ? r[st][e][c2] : 0u;
            const uint32_t lo01 = __builtin_amdgcn_perm(w[1], w[0], 0x05040100u);   // low halves of heads 0, 1
            const uint32_t lo23 = __builtin_amdgcn_perm(w[3], w[2], 0x05040100u);
            const uint32_t hi01 = __builtin_amdgcn_perm(w[1], w[0], 0x07060302u);   // high halves
            const uint32_t hi23 = __builtin_amdgcn_perm(w[3], w[2], 0x07060302u);
            trow[2 * ((t_lane + 2 * c2) ^ (t_dt & 7))] = u32x2{lo01, lo23};         // channel 2*c2
            trow[2 * ((t_lane + 2 * c2 + 1) ^ (t_dt & 7))] = u32x2{hi01, hi23};     // channel 2*c2 + 1
        }
        if (tid < 64) ld[buf][tid >> 5][(tid >> 4) & 1][tid & 15] = rf[st];
    };

    // pairs past the end are fetched as copies of the last one and never used
#pragma unroll
    for (int st = 0; st < kDepth; ++st) fetch(st, st);
    stash(0, 0);
    fetch(kDepth, 0);
    __syncthreads();
    // The trip count is rounded up to a multiple of kDepth and the steps past the end work on copies of
    // the last pair with every probability forced to zero: one loop exit, so the compiler's count of
    // loads still in flight is the same on every path into a step and its waits stay exact.
    for (int p0 = 0; p0 < n_pairs; p0 += kDepth) {
#pragma unroll
        for (int kk = 0; kk < kDepth; ++kk) {
            const int p = p0 + kk;
            const int cur = p & 1;
            const bool one = 2 * p < total, two = 2 * p + 1 < total;
            const int tk0 = seg * kSegTokens + list[min(2 * p, total - 1)], tk1 = seg * kSegTokens + list[min(2 * p + 1, total - 1)];
            const uint16_t *sq = stage[cur];
            bf16x8 ps, dss;                               // B operands of the second contractions
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int tok = u ? tk1 : tk0;
                f32x4 sacc = {0.f, 0.f, 0.f, 0.f}, dp = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 qa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&sq[(u * 16 + n) * kRowPitch + 32 * ks + 8 * g]));
                    const bf16x8 ga = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&sq[((2 + u) * 16 + n) * kRowPitch + 32 * ks + 8 * g]));
                    sacc = mfma16(qa, kB[ks], sacc);
                    dp = mfma16(ga, vB[ks], dp);
                }
                const float4 l4 = *reinterpret_cast<const float4 *>(&ld[cur][0][u][4 * g]);
                const float4 d4 = *reinterpret_cast<const float4 *>(&ld[cur][1][u][4 * g]);
                const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
                const bool dead = !(u ? two : one) || key > tok;   // padding past the end of the list; causal inside the own block
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    float pr = fast_exp2(__builtin_fmaf(sacc[rr], c, -ls[rr] * kLog2e));
                    if (dead || 4 * g + rr >= G || !(ls[rr] > -INFINITY)) pr = 0.f;
                    ps[4 * u + rr] = (__bf16)pr;
                    dss[4 * u + rr] = (__bf16)(pr * (dp[rr] - dl[rr]));
                }
            }
            // A operands of the second products: lane (n = channel, g), element 4u + e = (token u, head 4g + e)
            const u32x4 *tq = reinterpret_cast<const u32x4 *>(stageT[cur]);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                const u32x4 aq = tq[dt * 64 + (lane ^ (dt & 7))];
                const u32x4 ag = tq[(8 + dt) * 64 + (lane ^ (dt & 7))];
                dvT[dt] = mfma16(__builtin_bit_cast(bf16x8, ag), ps, dvT[dt]);
                dkT[dt] = mfma16(__builtin_bit_cast(bf16x8, aq), dss, dkT[dt]);
            }
            // pair p+1 goes to the other buffer (last read one step ago), its registers take pair p+1+kDepth
            constexpr int kD = kDepth;
            const int st = (kk + 1) % kD;
            __builtin_amdgcn_sched_barrier(0);            // keep the wait for this pair's registers behind the arithmetic
            stash(cur ^ 1, st);
            fetch(p + 1 + kD, st);
            __syncthreads();
        }
    }
    // ---- merge: lane holds channels 16*dt + 4*g .. +3 of its key --------------------------------------------
    if (key < L) {
        float *pk = acc_dk + (bh * dm.max_seqlen + key) * kHeadDim + 4 * g;
        float *pv = acc_dv + (bh * dm.max_seqlen + key) * kHeadDim + 4 * g;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                unsafeAtomicAdd(pk + 16 * dt + rr, dkT[dt][rr]);
                unsafeAtomicAdd(pv + 16 * dt + rr, dvT[dt][rr]);
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
    uint32_t *bitmap = reinterpret_cast<uint32_t *>(base + l.bitmap);
    float *acc_dk = reinterpret_cast<float *>(base + l.acc_dk), *acc_dv = reinterpret_cast<float *>(base + l.acc_dv);
    const int T = dm.max_seqlen;
    timing_begin("bwd_zero_kernel", stream);
    hipLaunchKernelGGL(bwd_zero_kernel, dim3(2048), dim3(256), 0, stream, reinterpret_cast<uint4 *>(base + l.zero_begin),
                       l.zero_bytes / sizeof(uint4));
    timing_end(stream);
    timing_begin("bwd_prep_kernel", stream);
    hipLaunchKernelGGL(bwd_prep_kernel, dim3((T + 3) / 4, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, out, dout,
                       seqlens, block_idx, delta, bitmap, l.nb_cap, l.words);
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
    if (bwd_seg_tokens(dm) == 4096)
        hipLaunchKernelGGL(attn_bwd_dkdv_kernel<4096>, dim3(l.nb_cap, l.words / 128, dm.batch * dm.Hkv), dim3(256), 0,
                           stream, dm, q, dout, kvb, l.nb_cap, seqlens, lse, delta, bitmap, l.words, acc_dk, acc_dv);
    else
        hipLaunchKernelGGL(attn_bwd_dkdv_kernel<2048>, dim3(l.nb_cap, l.words / 64, dm.batch * dm.Hkv), dim3(256), 0,
                           stream, dm, q, dout, kvb, l.nb_cap, seqlens, lse, delta, bitmap, l.words, acc_dk, acc_dv);
    timing_end(stream);
    timing_begin("bwd_finish_kernel", stream);
    hipLaunchKernelGGL(bwd_finish_kernel, dim3((T + 15) / 16, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, seqlens,
                       acc_dk, acc_dv, dk, dv);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
