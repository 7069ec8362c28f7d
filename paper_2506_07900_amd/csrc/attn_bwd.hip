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
static inline int bwd_seg_tokens(const Dims &dm) { return dm.max_seqlen > 65536 ? 4096 : 2048; }
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

// ---- dk, dv: a wavefront owns 32 keys of a block ---------------------------------------------------------
// 256 threads: a workgroup handles member tokens of block j that lie in one segment of the sequence (all of
// them, or one slice of the list when there are many).  The member tokens are compacted from the bitmap into a list
// and walked in pairs, two pairs per step.  Wave w owns the keys 64j + 32(w&1) .. +31 and, of their
// gradients, the channels 64(w>>1) .. +63: the two wavefronts of a key half both form S and dP of every
// pair (a wavefront that owned all 128 channels of dk and dv would need 128 accumulator registers on top
// of the 64 of its K and V operands, and spill).  With 32x32x16 MFMAs, rows = (token of the pair, head):
//   S  [row, key] = Q . K^T         A = the pair's q rows from LDS, B = K rows of the wave's keys (registers)
//   dP [row, key] = dO . V^T
//   dV^T[c, key] += dO^T[c, row] . P[row, key]      A = the same staged rows read through the transposing
//   dK^T[c, key] += Q^T [c, row] . dS[row, key]     LDS load, B = P / dS as they sit in the accumulators
// Staging: the 16 KiB of q and dout rows of a pair go from memory straight into LDS (no registers, no vector
// instructions), a step ahead of their use; two step buffers alternate.  They are two objects and the
// loop is unrolled by two, so that the compiler's wait counts let a read of one buffer run under the
// copies into the other.  A row is 256 bytes; its sixteen 16-byte pieces are stored XOR-swizzled with the
// head's two bit pairs exchanged: an operand load of the first products takes one piece from each of 16
// rows, a transposing load 32 bytes from each of 4 consecutive rows, and both then touch every bank once.
constexpr int kBwdSlices = 4;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
struct __align__(16) BwdRows {
    uint16_t rows[2][2][32][kHeadDim];                    // [pair of the step][q | dout][(token, head)][channel]: 32 KiB
};
struct __align__(16) BwdScalars {
    float ld[2][64];                                      // [pair][exponent offset of token a, of b | D of token a, of b][head]
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
    __shared__ BwdRows rows_even, rows_odd;
    __shared__ BwdScalars sc_even, sc_odd;
    __shared__ int total_s;
    // grid (segments x slices, blocks, B*Hkv): the initial blocks, which every token lists, come first in the
    // launch order; a (block, segment) unit with many members is shared by up to kBwdSlices workgroups, each
    // taking kSliceTokens consecutive members (the time of the longest workgroup bounds the kernel otherwise)
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
    const int n_steps = (total + 3) >> 2;                 // four tokens per step
    const int kh = wave & 1, chh = wave >> 1;             // key half; channel half of the gradients
    const int c32 = lane & 31, hf = lane >> 5;
    // ---- this wave's keys as B operands: lane (c32, hf) = key 32kh + c32, channels 16ks + 8hf .. +7, picked
    // out of the 16-key fragments of the packed block ------------------------------------------------------
    const u32x4 *blk = reinterpret_cast<const u32x4 *>(kvb) + (bh * nb_cap + j) * kBwdBlockU4;
    bf16x8 kB[8], vB[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const int at = ((ks >> 1) * 4 + 2 * kh + (c32 >> 4)) * 64 + (2 * (ks & 1) + hf) * 16 + (c32 & 15);
        kB[ks] = __builtin_bit_cast(bf16x8, blk[at]);
        vB[ks] = __builtin_bit_cast(bf16x8, blk[1024 + at]);
    }
    f32x16 dkT[2], dvT[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) dkT[ct][v] = dvT[ct][v] = 0.f;
    const int key = j * kBlock + 32 * kh + c32;           // this lane's key (column of S)

    // staging: wave w copies heads 4w .. 4w+3 of both tokens of a pair, q and dout: four 1 KiB copies per pair,
    // lane = (head 4w + lane/16, piece lane%16 of the LDS row = piece (lane%16) ^ head of the row in memory)
    const int s_n = 4 * wave + (lane >> 4);
    const int s_piece = (lane & 15) ^ bwd_swizzle(s_n);
    const __bf16 *s_q = q.ptr + b * q.sb + (int64_t)(h * G + min(s_n, G - 1)) * q.sh + 8 * s_piece;
    const __bf16 *s_g = dout.ptr + b * dout.sb + (int64_t)(h * G + min(s_n, G - 1)) * dout.sh + 8 * s_piece;
    const float *s_f = rowc + ((int64_t)b * dm.max_seqlen * dm.Hkv + h) * 32 + 16 * (lane >> 5) + (lane & 15);   // + 32 Hkv tok
    auto stage = [&](BwdRows &dst, BwdScalars &dsc, int s) __attribute__((always_inline)) {
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            const int p = 2 * s + pr;                     // pairs past the end are copies of the last token, never used
            const int ta = seg * kSegTokens + list[min(2 * p, total - 1)], tb = seg * kSegTokens + list[min(2 * p + 1, total - 1)];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int part = k >> 1, u = k & 1;
                const int tok = u ? tb : ta;
                const __bf16 *src = part ? s_g + (int64_t)tok * dout.st : s_q + (int64_t)tok * q.st;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)&dst.rows[pr][part][16 * u + 4 * wave][0],
                                                 16, 0, 0);
            }
            if (wave == 0) {
                const int tok = ((lane >> 4) & 1) ? tb : ta;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(s_f + (int64_t)tok * dm.Hkv * 32),
                                                 (__attribute__((address_space(3))) void *)&dsc.ld[pr][0], 4, 0, 0);
            }
        }
    };
    // LDS addresses of the operand loads, the parts that depend on the lane
    const uint32_t a_row = (uint32_t)c32 * 256u + (uint32_t)((hf ^ bwd_swizzle(c32 & 15)) << 4);   // piece 2ks + hf of row c32: ^ (ks << 5)
    const uint32_t t_r = 4u * hf + ((lane & 15) >> 2), t_c = 2u * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    // (channel tile 2chh + ct starts at piece 8chh + 4ct; rows 8rd + t_r have swizzle 2rd ^ swizzle(t_r))
    const uint32_t a_tr = t_r * 256u + ((t_c ^ (uint32_t)bwd_swizzle((int)t_r) ^ (8u * chh)) << 4) + 8u * (lane & 1);   // ^ ((4ct ^ 2rd) << 4), + (16 s2 + 8 rd) rows

    auto compute = [&](const BwdRows &cur, const BwdScalars &csc, int s, int pp) __attribute__((always_inline)) {
        const int p = 2 * s + pp;
        const bool one = 2 * p < total, two = 2 * p + 1 < total;
        const int tk0 = seg * kSegTokens + list[min(2 * p, total - 1)], tk1 = seg * kSegTokens + list[min(2 * p + 1, total - 1)];
        const char *xq = reinterpret_cast<const char *>(&cur.rows[pp][0][0][0]);
        const char *xg = reinterpret_cast<const char *>(&cur.rows[pp][1][0][0]);
        f32x16 sacc, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = dp[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const u32x4 qa = *reinterpret_cast<const u32x4 *>(xq + (a_row ^ (uint32_t)(ks << 5)));
            const u32x4 ga = *reinterpret_cast<const u32x4 *>(xg + (a_row ^ (uint32_t)(ks << 5)));
            sacc = mfma32(__builtin_bit_cast(bf16x8, qa), kB[ks], sacc);
            dp = mfma32(__builtin_bit_cast(bf16x8, ga), vB[ks], dp);
        }
        // accumulator entry v of a lane: row 8(v/4) + 4hf + v%4 = (token v/8, head 8((v/4)%2) + 4hf + v%4), column = key.
        // Padding of the list and the causal edge inside the own block: the exponent's offset becomes -inf.
        const float bias0 = (!one | (key > tk0)) ? -INFINITY : 0.f, bias1 = (!two | (key > tk1)) ? -INFINITY : 0.f;
        bf16x8 ps[2], dss[2];                             // B operands of the second products, one k-step per token
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
            const float4 n4 = *reinterpret_cast<const float4 *>(&csc.ld[pp][8 * j4 + 4 * hf]);
            const float4 d4 = *reinterpret_cast<const float4 *>(&csc.ld[pp][32 + 8 * j4 + 4 * hf]);
            const float nl[4] = {n4.x, n4.y, n4.z, n4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
            const float bias = (j4 >> 1) ? bias1 : bias0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int v = 4 * j4 + e;
                const float pr = fast_exp2(__builtin_fmaf(sacc[v], c, nl[e] + bias));
                ps[v >> 3][v & 7] = (__bf16)pr;
                dss[v >> 3][v & 7] = (__bf16)(pr * (dp[v] - dl[e]));
            }
        }
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const uint32_t o0 = (a_tr ^ (uint32_t)((4 * ct) << 4)) + (uint32_t)(16 * s2) * 256u;
                const uint32_t o1 = (a_tr ^ (uint32_t)(((4 * ct) ^ 2) << 4)) + (uint32_t)(16 * s2 + 8) * 256u;
                const s16x4 g0 = lds_read_tr16(xg + o0), g1 = lds_read_tr16(xg + o1);
                const s16x4 q0 = lds_read_tr16(xq + o0), q1 = lds_read_tr16(xq + o1);
                const bf16x8 ag = __builtin_bit_cast(bf16x8, __builtin_shufflevector(g0, g1, 0, 1, 2, 3, 4, 5, 6, 7));
                const bf16x8 aq = __builtin_bit_cast(bf16x8, __builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7));
                dvT[ct] = mfma32(ag, ps[s2], dvT[ct]);
                dkT[ct] = mfma32(aq, dss[s2], dkT[ct]);
            }
    };
    auto step = [&](BwdRows &cur, BwdScalars &csc, BwdRows &nxt, BwdScalars &nsc, int s) __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(0);                    // this wavefront's copies for step s have landed
        __syncthreads();                                  // everyone's have, and everyone is past its reads of step s - 1
        if (s + 1 < n_steps) stage(nxt, nsc, s + 1);
        compute(cur, csc, s, 0);
        if (2 * (2 * s + 1) < total) compute(cur, csc, s, 1);   // (uniform)
    };
    stage(rows_even, sc_even, 0);
    for (int s = 0; s < n_steps; s += 2) {
        step(rows_even, sc_even, rows_odd, sc_odd, s);
        if (s + 1 < n_steps) step(rows_odd, sc_odd, rows_even, sc_even, s + 1);
    }
    // ---- merge: a lane holds channels 64chh + 32ct + 8(v/4) + 4hf + v%4 of its key.  The tiles are turned through
    // LDS (the staging buffers, 8 KiB per wavefront) so that one atomic instruction covers 64 consecutive
    // channels of one key: two cache lines instead of 64. ------------------------------------------------------
    __syncthreads();                                      // every wavefront is past its last read of the staging buffers
    float *tile = reinterpret_cast<float *>(wave < 2 ? &rows_even.rows[0][0][0][0] : &rows_odd.rows[0][0][0][0]) + (wave & 1) * 2048;
    const int key0 = j * kBlock + 32 * kh;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        float *acc = (which ? acc_dv : acc_dk) + (bh * dm.max_seqlen + key0) * kHeadDim + 64 * chh + lane;
        // [key][16-byte piece ^ (key & 15)][4 channels]
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const f32x16 &t = which ? dvT[ct] : dkT[ct];
                const int piece = 8 * ct + 2 * v4 + hf;   // channels 4 piece .. +3 of the wave's 64
                *reinterpret_cast<float4 *>(tile + c32 * 64 + ((piece ^ (c32 & 15)) << 2)) =
                    float4{t[4 * v4], t[4 * v4 + 1], t[4 * v4 + 2], t[4 * v4 + 3]};
            }
        // (same wavefront wrote and reads: LDS keeps the order)
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            const float x = tile[k * 64 + ((((lane >> 2) ^ (k & 15)) << 2) | (lane & 3))];
            if (key0 + k < L) unsafeAtomicAdd(acc + (int64_t)k * kHeadDim, x);
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
    if (bwd_seg_tokens(dm) == 4096)
        hipLaunchKernelGGL(attn_bwd_dkdv_kernel<4096>, dim3(l.nb_cap, l.words / 128 * kBwdSlices, dm.batch * dm.Hkv), dim3(256), 0,
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
