// Stage 2, prefill, for G = 16 query heads per key-value head (the group size the paper
// recommends, "Hyper-Parameter Recommendation"): one query token's head group is exactly one
// 16-row MFMA tile.  Same mathematics as select_prefill.hip, organised for the matrix cores:
//
//   pack_ck_kernel        compressed keys -> fragment-major copy (a wavefront reads the operand
//                         of one 16-kernel tile as four coalesced 1 KiB loads, no LDS)
//   select_lse16_kernel   pass 1: log-sum-exp of every (token, head) row over its visible kernels
//   select_score16_kernel pass 2: scores 2^(z - lse), mean over the 16 heads, 5-wide / stride-4
//                         max over kernels -> block scores of the candidate blocks
// followed by select_pick_kernel (select_prefill.hip), the row-parallel top-k.
//
// A wavefront owns 8 consecutive tokens and works alone (no LDS, no barriers).  MFMA and plain
// VALU work only overlap on this hardware when they alternate inside one instruction stream, so
// both passes are software-pipelined by hand: the MFMAs of kernel tile t are issued in the same
// basic block as the exponentials / reductions of tile t-1.
#include "common.h"

namespace infllmv2 {

constexpr int kMT = 8;                 // tokens (= 16-row tiles) per wavefront
constexpr int kTokPerWg16 = 4 * kMT;   // 4 independent wavefronts per workgroup

__device__ inline int n_visible16(int i) { return num_kernels(i + 1); }
// kernels of pass 1: the fine ones, or the coarse ones of the approximate log-sum-exp
__device__ inline int n_visible_lse(int i, int rho) {
    const int nf = num_kernels(i + 1);
    return rho > 1 ? num_coarse(nf, rho) : nf;
}

// DPP helpers on floats (row = 16 lanes).  Lanes whose source falls outside the row keep `old`.
template <int kCtrl>
__device__ inline float dpp_f32(float old, float src) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old),
                                                                  __builtin_bit_cast(int, src), kCtrl,
                                                                  0xf, 0xf, false));
}
constexpr int kRowShl1 = 0x101, kRowShl2 = 0x102, kRowShr1 = 0x111, kRowRor1 = 0x121;

// ---- compressed keys -> fragment-major ------------------------------------------------------------
// tile t (kernels 16t..16t+15), k-step ks, lane (g, n):  CK[16t + n][32ks + 8g .. +7]; 4 KiB per tile.
__global__ __launch_bounds__(256) void pack_ck_kernel(Dims dm, Tensor ck, const int32_t *__restrict__ seqlens,
                                                       uint4 *__restrict__ ckp, int32_t nt_cap) {
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int n_c = num_kernels(L);
    if (16 * t >= n_c) return;
    const int c = threadIdx.x, ks = c >> 6, lane = c & 63, n = lane & 15, g = lane >> 4;
    uint4 x = {0u, 0u, 0u, 0u};
    if (16 * t + n < n_c)
        x = *reinterpret_cast<const uint4 *>(ck.ptr + b * ck.sb + h * ck.sh + (int64_t)(16 * t + n) * ck.st +
                                             32 * ks + 8 * g);
    ckp[(((int64_t)b * dm.Hkv + h) * nt_cap + t) * 256 + c] = x;
}

// Coarse kernels of the approximate log-sum-exp ("Efficient Top-K Implementation", last
// paragraph), built from the fine representations and stored fragment-major like them:
// CKc[c] = bf16(mean_r CK[rho*c + 2r]), r < rho.  The sum of rho bf16 values is exact in fp64, so
// the result is the correctly rounded mean.
__global__ __launch_bounds__(256) void pack_ck_coarse_kernel(Dims dm, Tensor ck, const int32_t *__restrict__ seqlens,
                                                              uint4 *__restrict__ ckp, int32_t nt_cap) {
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int n_cc = num_coarse(num_kernels(L), dm.rho);
    if (16 * t >= n_cc) return;
    const int c = threadIdx.x, ks = c >> 6, lane = c & 63, n = lane & 15, g = lane >> 4;
    uint4 x = {0u, 0u, 0u, 0u};
    const int cc = 16 * t + n;
    if (cc < n_cc) {
        double acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.0;
        for (int r = 0; r < dm.rho; ++r) {
            const bf16x8 v = load8(ck.ptr + b * ck.sb + h * ck.sh + (int64_t)(dm.rho * cc + 2 * r) * ck.st +
                                   32 * ks + 8 * g);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (double)(float)v[e];
        }
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)f64_to_bf16_rne(acc[2 * e] / (double)dm.rho) |
                   ((uint32_t)f64_to_bf16_rne(acc[2 * e + 1] / (double)dm.rho) << 16);
        x = uint4{w[0], w[1], w[2], w[3]};
    }
    ckp[(((int64_t)b * dm.Hkv + h) * nt_cap + t) * 256 + c] = x;
}

struct Frag4 {
    uint4 f[4];
};
__device__ inline Frag4 load_ck_tile(const uint4 *ckp_head, int t, int lane) {
    Frag4 r;
    const uint4 *p = ckp_head + (int64_t)t * 256 + lane;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) r.f[ks] = p[ks * 64];
    return r;
}

__device__ inline void load_q16(bf16x8 (&qf)[kMT][4], const Tensor &q, int b, int h, int t0, int L, int n, int g) {
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
        const int tok = t0 + mt;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[mt][ks] = zero8();
            if (tok < L)
                qf[mt][ks] = load8(q.ptr + b * q.sb + (int64_t)tok * q.st + (int64_t)(h * 16 + n) * q.sh +
                                   32 * ks + 8 * g);
        }
    }
}

// ---- shared pieces of the two passes -------------------------------------------------------------------
// The 8 tokens of a wavefront are handled as two halves of 4 (A: tokens 0..3, B: 4..7) that
// ping-pong: while the matrix cores work on one half of kernel tile t, the vector ALU finishes the
// other half's previous results, inside one basic block.
constexpr int kHalf = 4;

// 16 MFMAs: logits of one 16-kernel tile against 4 tokens.  kKeysAreRows picks the orientation:
//   true   Z^T = CK . Q^T   lane = (head n), accumulator entries = kernels 4g..4g+3
//   false  Z   = Q . CK^T   lane = (kernel n), accumulator entries = heads 4g..4g+3
template <bool kKeysAreRows>
__device__ inline void mfma_half(const Frag4 &fr, const bf16x8 (&qf)[kMT][4], int base, f32x4 (&z)[kHalf]) {
#pragma unroll
    for (int u = 0; u < kHalf; ++u) z[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int u = 0; u < kHalf; ++u) {
            const bf16x8 ckf = __builtin_bit_cast(bf16x8, fr.f[ks]);
            z[u] = kKeysAreRows ? mfma16(ckf, qf[base + u][ks], z[u]) : mfma16(qf[base + u][ks], ckf, z[u]);
        }
}

// ---- pass 1 ------------------------------------------------------------------------------------------
// Lane = one (token, head) row; it sums 2^(z*c - m_ref) over its own kernels (4 per tile) and the
// four 16-lane groups are merged at the end.  m_ref is a logit of the row itself, re-based only
// when a partial sum leaves the safe range, so the common path has no max tracking at all:
// neg_m = -m_ref starts as NaN, which sends the first tile through the re-basing path.
__global__ __launch_bounds__(256, 2) void select_lse16_kernel(Dims dm, Tensor q, const uint4 *__restrict__ ckp,
                                                            int32_t nt_cap, const int32_t *__restrict__ seqlens,
                                                            float *__restrict__ lse2, int32_t n_tiles) {
    const int tile = n_tiles - 1 - (int)(blockIdx.x % n_tiles);       // longest rows first
    const int h = (blockIdx.x / n_tiles) % dm.Hkv;
    const int b = blockIdx.x / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = tile * kTokPerWg16 + wave * kMT;
    if (t0 >= L) return;
    const int n = lane & 15, g = lane >> 4;
    const float c = dm.scale_log2;

    bf16x8 qf[kMT][4];
    load_q16(qf, q, b, h, t0, L, n, g);
    float neg_m[kMT], s_run[kMT];
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
        neg_m[mt] = __builtin_nanf("");
        s_run[mt] = 0.f;
    }
    const int last_tok = min(t0 + kMT, (int)L) - 1;
    const int nvis_hi = n_visible_lse(last_tok, dm.rho), nvis_lo = n_visible_lse(t0, dm.rho);
    const int nt_full = nvis_lo >> 4;                    // tiles wholly visible to every token here
    const int nt_all = (nvis_hi + 15) >> 4;
    const uint4 *ckp_head = ckp + ((int64_t)b * dm.Hkv + h) * nt_cap * 256;

    auto finish = [&](const f32x4 (&z)[kHalf], int base) {
        float acc[kHalf];
        bool bad = false;
#pragma unroll
        for (int u = 0; u < kHalf; ++u) {
            float a = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) a += fast_exp2(__builtin_fmaf(z[u][j], c, neg_m[base + u]));
            acc[u] = a;
            bad |= !(a <= 0x1p60f);                      // too large, inf, or NaN (no reference yet)
        }
        if (__any(bad)) {                                // rare: re-base on this tile's own maximum
#pragma unroll
            for (int u = 0; u < kHalf; ++u)
                if (!(acc[u] <= 0x1p60f)) {
                    const float tmax = fmaxf(fmaxf(z[u][0], z[u][1]), fmaxf(z[u][2], z[u][3])) * c;
                    if (tmax > -INFINITY) {
                        const float old = neg_m[base + u];
                        s_run[base + u] = (old != old) ? 0.f : s_run[base + u] * fast_exp2(-old - tmax);
                        neg_m[base + u] = -tmax;
                        float a = 0.f;
#pragma unroll
                        for (int j = 0; j < 4; ++j) a += fast_exp2(__builtin_fmaf(z[u][j], c, -tmax));
                        acc[u] = a;
                    } else {
                        acc[u] = 0.f;                    // every kernel of this lane masked so far
                    }
                }
        }
#pragma unroll
        for (int u = 0; u < kHalf; ++u) s_run[base + u] += acc[u];
    };

    f32x4 zA[kHalf], zB[kHalf];
    if (nt_full > 0) {
        // two fragment buffers that swap roles each tile (the loop is unrolled by two so that no
        // register copies are needed): one feeds the matrix cores, the other receives the next tile
        Frag4 f0 = load_ck_tile(ckp_head, 0, lane);
        Frag4 f1 = f0;
        if (nt_full > 1) f1 = load_ck_tile(ckp_head, 1, lane);
        mfma_half<true>(f0, qf, 0, zA);
        mfma_half<true>(f0, qf, kHalf, zB);
        finish(zA, 0);
        auto tile_step = [&](const Frag4 &f) {
            mfma_half<true>(f, qf, 0, zA);               // matrix work on half A of this tile ...
            finish(zB, kHalf);                           // ... alternates with half B of the previous tile
            mfma_half<true>(f, qf, kHalf, zB);
            finish(zA, 0);
        };
        int t = 1;
        for (; t + 1 < nt_full; t += 2) {
            f0 = load_ck_tile(ckp_head, t + 1, lane);
            tile_step(f1);
            if (t + 2 < nt_full) f1 = load_ck_tile(ckp_head, t + 2, lane);
            tile_step(f0);
        }
        if (t < nt_full) tile_step(f1);
        finish(zB, kHalf);
    }
    for (int t = nt_full; t < nt_all; ++t) {             // causal edge: at most two masked tiles
        const Frag4 fr = load_ck_tile(ckp_head, t, lane);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            mfma_half<true>(fr, qf, half * kHalf, zA);
#pragma unroll
            for (int u = 0; u < kHalf; ++u) {
                const int nv = n_visible_lse(t0 + half * kHalf + u, dm.rho);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (16 * t + 4 * g + j >= nv) zA[u][j] = -INFINITY;
            }
            finish(zA, half * kHalf);
        }
    }
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
        const float m_lane = (neg_m[mt] != neg_m[mt]) ? -INFINITY : -neg_m[mt];
        const float M = xgroup_max(m_lane);
        const float m_use = M == -INFINITY ? 0.f : M;
        const float S = xgroup_sum(s_run[mt] * fast_exp2(m_lane - m_use));
        const int tok = t0 + mt;
        float lse = M + fast_log2(S);
        // approximate mode: rho times fewer kernels were summed (log2 rho is an integer); a query
        // that sees no coarse kernel yet gets 0 (it has no candidate blocks to rank)
        if (dm.rho > 1) lse = M == -INFINITY ? 0.f : lse + (float)(31 - __clz(dm.rho));
        if (g == 0 && tok < L) lse2[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * 16 + n] = lse;
    }
}

// ---- pass 2 ----------------------------------------------------------------------------------------
// Lane = kernel n of the tile, accumulator entries = heads 4g..4g+3 of the token.  The block scores
// never leave the compute unit: the wavefront keeps the scores of its 8 tokens for a chunk of 64*VPL
// key-value blocks in LDS, and at the end of a chunk merges them into each token's running top
// n_pick (wave_topk over the chunk's scores plus the carried picks), so the selection costs no score
// matrix and no second kernel.  After the last chunk the forced blocks are added and the row written.
// VPL = 0: the scores R[token, j] of the candidate blocks go to memory instead (-inf when no visible
// kernel intersects the block); only the query-block-shared comparison variant, which averages them
// over 64 tokens before ranking, uses that.
struct Score16Lds {                                      // layout of one wavefront's piece of LDS
    int chunk_blocks, carry_words, topk_words;
    __host__ __device__ Score16Lds(int vpl, int topk)
        : chunk_blocks(64 * vpl), carry_words(kMT * ((topk + 1) & ~1)),
          topk_words(64 + topk_cand_cap(topk, vpl + 1)) {}
    __host__ __device__ size_t bytes() const {
        return (size_t)kMT * chunk_blocks * sizeof(float) + (size_t)(carry_words + topk_words) * sizeof(uint64_t) +
               kMT * 16 * sizeof(float);
    }
};

template <int VPL>
__global__ __launch_bounds__(256, 2) void select_score16_kernel(Dims dm, Tensor q, const uint4 *__restrict__ ckp,
                                                              int32_t nt_cap, const int32_t *__restrict__ seqlens,
                                                              const float *__restrict__ lse2,
                                                              float *__restrict__ R, int32_t nb_cap,
                                                              int32_t n_tiles, int32_t *__restrict__ block_idx) {
    extern __shared__ __align__(16) unsigned char score_smem[];
    constexpr bool kFused = VPL > 0;
    constexpr int kChunkBlocks = 64 * VPL;
    constexpr int kChunkTiles = kFused ? kChunkBlocks / 4 : (1 << 30);
    const int tile = n_tiles - 1 - (int)(blockIdx.x % n_tiles);
    const int h = (blockIdx.x / n_tiles) % dm.Hkv;
    const int b = blockIdx.x / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = tile * kTokPerWg16 + wave * kMT;
    if (t0 >= L) return;
    const int n = lane & 15, g = lane >> 4;
    const float c = dm.scale_log2;

    // the 8 tokens share their own block (8 divides 64), hence the candidate range and the counts
    const int b_own = t0 / kBlock, n_blk = b_own + 1;
    const int n_init = dm.n_init < n_blk ? dm.n_init : n_blk;
    const int lo_local = max(n_init, b_own - dm.n_local + 1);                 // forced trailing: lo_local..b_own
    const int jc_max = lo_local - 1;                                          // candidates: n_init..jc_max
    const int n_sel = dm.topk < n_blk ? dm.topk : n_blk;
    const int n_pick = n_sel - (n_init + (b_own - jc_max));
    const int64_t row0 = ((int64_t)b * dm.Hkv + h) * dm.max_seqlen + t0;
    const Score16Lds lay(VPL, dm.topk);
    float *Rl = reinterpret_cast<float *>(score_smem + (size_t)wave * lay.bytes());   // [kMT][kChunkBlocks]
    uint64_t *carry = reinterpret_cast<uint64_t *>(Rl + kMT * kChunkBlocks);          // [kMT][carry_words / kMT]
    uint64_t *tk_lds = carry + lay.carry_words;
    const int carry_pitch = lay.carry_words / kMT;
    const int nt_all = (n_pick > 0 && jc_max >= n_init) ? min((4 * jc_max + 4 + 15) >> 4, nt_cap) : 0;
    if (!kFused && nt_all <= 0) return;                                       // forced blocks only

    if (nt_all > 0) {
        bf16x8 qf[kMT][4];
        load_q16(qf, q, b, h, t0, L, n, g);
        float *nls = reinterpret_cast<float *>(tk_lds + lay.topk_words);    // [kMT][16]: -lse of head, token
        for (int i = lane; i < kMT * 16; i += 64)
            nls[i] = (t0 + (i >> 4) < L) ? -lse2[((int64_t)b * dm.max_seqlen + t0 + (i >> 4)) * dm.Hq + h * 16 + (i & 15)] : 0.f;
        __builtin_amdgcn_wave_barrier();
        const int nt_pipe = min(n_visible16(t0) >> 4, nt_all);                // tiles needing no mask
        const uint4 *ckp_head = ckp + ((int64_t)b * dm.Hkv + h) * nt_cap * 256;
        // packed per-token values: 16-lane group g of half i belongs to token 4i+g
        float prev_v[2] = {-INFINITY, -INFINITY};
        float *Rrow[2];
        bool wr[2];
        int nvis_tok[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int tok = t0 + 4 * i + g;
            Rrow[i] = kFused ? Rl + (4 * i + g) * kChunkBlocks + (n >> 2) : R + (row0 + 4 * i + g) * nb_cap + (n >> 2);
            wr[i] = ((n & 3) == 0) && tok < L;
            nvis_tok[i] = n_visible16(tok);
        }
        if (kFused)
            for (int i = lane; i < lay.carry_words; i += 64) carry[i] = 0ull;

        // epilogue of tile t for half i: 2^(z*c - lse), sum over the 16 heads, mean, floor, causal mask,
        // 5-wide / stride-4 max over kernels -> lanes n = 0,4,8,12 hold blocks 4t + n/4
        auto finish = [&](const f32x4 (&z)[kHalf], int i, int t) {
            float e[kHalf];
#pragma unroll
            for (int u = 0; u < kHalf; ++u) {
                float a = 0.f;
                const f32x4 nl4 = *reinterpret_cast<const f32x4 *>(nls + (kHalf * i + u) * 16 + 4 * g);
#pragma unroll
                for (int j = 0; j < 4; ++j) a += fast_exp2(__builtin_fmaf(z[u][j], c, nl4[j]));
                e[u] = a;
            }
            // sum over the four 16-lane groups, leaving token u's total in group u (3 lane swaps)
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            const v2u p01 = __builtin_amdgcn_permlane16_swap(__float_as_uint(e[0]), __float_as_uint(e[1]), false, false);
            const v2u p23 = __builtin_amdgcn_permlane16_swap(__float_as_uint(e[2]), __float_as_uint(e[3]), false, false);
            const float s01 = __uint_as_float(p01[0]) + __uint_as_float(p01[1]);
            const float s23 = __uint_as_float(p23[0]) + __uint_as_float(p23[1]);
            const v2u pq = __builtin_amdgcn_permlane32_swap(__float_as_uint(s01), __float_as_uint(s23), false, false);
            float v = __uint_as_float(pq[0]) + __uint_as_float(pq[1]);
            v = fminf(fmaxf(v * (1.f / 16.f), kScoreFloor), kScoreCeil);
            if (t >= nt_pipe && 16 * t + n >= nvis_tok[i]) v = -INFINITY;     // kernel not visible to this token
            const float a = fmaxf(v, dpp_f32<kRowShl1>(v, v));
            const float bq = fmaxf(a, dpp_f32<kRowShl2>(a, a));
            const float halo0 = dpp_f32<kRowRor1>(prev_v[i], prev_v[i]);      // lane 0 <- previous tile's lane 15
            const float halo = dpp_f32<kRowShr1>(halo0, v);                   // lane n <- v[n-1]
            const float w = fmaxf(bq, halo);
            prev_v[i] = v;
            if (kFused) {
                if (wr[i]) Rrow[i][(4 * t) & (kChunkBlocks - 1)] = w;
            } else {
                const int j = 4 * t + (n >> 2);
                if (wr[i] && j >= n_init && j <= jc_max) Rrow[i][4 * t] = w;
            }
        };

        // the tiles [ta, te) through the software pipeline
        auto run_tiles = [&](int ta, int te) {
            f32x4 zA[kHalf], zB[kHalf];
            // two fragment buffers that swap roles each tile (loop unrolled by two: no register copies)
            Frag4 f0 = load_ck_tile(ckp_head, ta, lane);
            Frag4 f1 = f0;
            if (ta + 1 < te) f1 = load_ck_tile(ckp_head, ta + 1, lane);
            mfma_half<false>(f0, qf, 0, zA);
            mfma_half<false>(f0, qf, kHalf, zB);
            finish(zA, 0, ta);
            auto tile_step = [&](const Frag4 &f, int t) {
                mfma_half<false>(f, qf, 0, zA);              // matrix work on half A of tile t ...
                finish(zB, 1, t - 1);                        // ... alternates with the epilogue of half B, tile t-1
                mfma_half<false>(f, qf, kHalf, zB);
                finish(zA, 0, t);
            };
            int t = ta + 1;
            for (; t + 1 < te; t += 2) {
                f0 = load_ck_tile(ckp_head, t + 1, lane);
                tile_step(f1, t);
                if (t + 2 < te) f1 = load_ck_tile(ckp_head, t + 2, lane);
                tile_step(f0, t + 1);
            }
            if (t < te) tile_step(f1, t);
            finish(zB, 1, te - 1);
        };

        for (int ta = 0; ta < nt_all; ta += kChunkTiles) {
            run_tiles(ta, min(ta + kChunkTiles, nt_all));
            if (kFused) {                                                     // merge the chunk into the running picks
                __builtin_amdgcn_wave_barrier();
                const int j0 = 4 * ta;
                for (int u = 0; u < kMT && t0 + u < L; ++u) {
                    constexpr int NE = kFused ? VPL + 1 : 1;
                    uint64_t el[NE];
#pragma unroll
                    for (int s2 = 0; s2 < NE - 1; ++s2)
                        el[s2] = pick_element(Rl[u * kChunkBlocks + lane + 64 * s2], j0 + lane + 64 * s2, n_init, jc_max);
                    el[NE - 1] = lane < n_pick ? carry[u * carry_pitch + lane] : 0ull;
                    const uint64_t res = wave_topk<NE>(el, n_pick, tk_lds, lane);
                    if (lane < n_pick) carry[u * carry_pitch + lane] = res;
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
    if (kFused) {
        for (int u = 0; u < kMT && t0 + u < L; ++u) {
            const int picked = (nt_all > 0 && lane < n_pick) ? (int)~(uint32_t)carry[u * carry_pitch + lane] : 0;
            write_block_row(picked, n_pick > 0 ? n_pick : 0, n_sel, n_init, lo_local, dm.topk,
                            block_idx + (row0 + u) * dm.topk, lane);
        }
    }
}

// Tiles of 16 fine kernels in the fragment-major copy: those that hold a kernel of the longest sequence,
// plus one.  A token's last candidate block can lie one tile past the last kernel of its sequence (none
// of that tile's kernels is visible, but the block's left-neighbour kernel in the tile before can be), and
// pass 2 walks that tile like any other: its loads have to stay inside the buffer, whatever they return.
static int32_t fine_tiles_cap(const Dims &dm) { return (num_kernels(dm.max_seqlen) + 15) / 16 + 1; }
static int32_t coarse_tiles_cap(const Dims &dm) {
    return dm.rho > 1 ? (num_coarse(num_kernels(dm.max_seqlen), dm.rho) + 15) / 16 : 0;
}
static size_t coarse_tiles_bytes(const Dims &dm) {
    const size_t b = (size_t)dm.batch * dm.Hkv * coarse_tiles_cap(dm) * 256 * sizeof(uint4);
    return (b + 255) / 256 * 256;
}

// Key-value blocks per chunk of the in-kernel top-k, in units of 64: the whole row in one chunk when it
// fits, and never more LDS than lets two workgroups share a compute unit.
static int score16_vpl(const Dims &dm) {
    const int n_blocks = (dm.max_seqlen + kBlock - 1) / kBlock;
    int vpl = n_blocks <= 128 ? 2 : n_blocks <= 256 ? 4 : 8;
    while (vpl > 2 && 4 * Score16Lds(vpl, dm.topk).bytes() > 80 * 1024) vpl /= 2;
    return vpl;
}

size_t select_prefill16_ws_bytes(const Dims &dm) {
    size_t lse = (size_t)dm.batch * dm.max_seqlen * dm.Hq * sizeof(float);
    lse = (lse + 255) / 256 * 256;
    const size_t nt_cap = (size_t)fine_tiles_cap(dm);
    size_t ckp = (size_t)dm.batch * dm.Hkv * nt_cap * 256 * sizeof(uint4);
    ckp = (ckp + 255) / 256 * 256;
    return lse + ckp + coarse_tiles_bytes(dm) + select_scores_bytes(dm) + select_shared_scores_bytes(dm);
}

int launch_select_prefill16(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens, int32_t *block_idx,
                            void *ws, hipStream_t stream, float *scores_out, int32_t scores_pitch) {
    size_t lse_bytes = (size_t)dm.batch * dm.max_seqlen * dm.Hq * sizeof(float);
    lse_bytes = (lse_bytes + 255) / 256 * 256;
    const int32_t nt_cap = fine_tiles_cap(dm);
    size_t ckp_bytes = (size_t)dm.batch * dm.Hkv * nt_cap * 256 * sizeof(uint4);
    ckp_bytes = (ckp_bytes + 255) / 256 * 256;
    float *lse2 = reinterpret_cast<float *>(ws);
    uint4 *ckp = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(ws) + lse_bytes);
    uint4 *ckp_c = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(ws) + lse_bytes + ckp_bytes);
    const int32_t ntc_cap = coarse_tiles_cap(dm);
    float *R = scores_out ? scores_out
                          : reinterpret_cast<float *>(reinterpret_cast<char *>(ws) + lse_bytes + ckp_bytes + coarse_tiles_bytes(dm));
    const int32_t nb_cap = scores_out ? scores_pitch : select_scores_pitch(dm);
    const int32_t n_tiles = (dm.max_seqlen + kTokPerWg16 - 1) / kTokPerWg16;
    const int64_t n_wg = (int64_t)n_tiles * dm.Hkv * dm.batch;
    if (n_wg <= 0) return 0;
    if (nt_cap > 0) {
        timing_begin("pack_ck_kernel", stream);
        hipLaunchKernelGGL(pack_ck_kernel, dim3(nt_cap, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, ck, seqlens,
                           ckp, nt_cap);
        timing_end(stream);
        if (dm.rho > 1 && ntc_cap > 0) {                 // pass 1 runs over the coarse kernels
            timing_begin("pack_ck_coarse_kernel", stream);
            hipLaunchKernelGGL(pack_ck_coarse_kernel, dim3(ntc_cap, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, ck,
                               seqlens, ckp_c, ntc_cap);
            timing_end(stream);
        }
        timing_begin("select_lse16_kernel", stream);
        hipLaunchKernelGGL(select_lse16_kernel, dim3((uint32_t)n_wg), dim3(256), 0, stream, dm, q,
                           dm.rho > 1 ? ckp_c : ckp, dm.rho > 1 ? ntc_cap : nt_cap, seqlens, lse2, n_tiles);
        timing_end(stream);
        timing_begin("select_score16_kernel", stream);
        if (dm.shared_q || scores_out) {
            hipLaunchKernelGGL(select_score16_kernel<0>, dim3((uint32_t)n_wg), dim3(256),
                               4 * Score16Lds(0, dm.topk).bytes(), stream, dm, q, ckp, nt_cap, seqlens, lse2, R, nb_cap,
                               n_tiles, block_idx);
        } else {
            const int vpl = score16_vpl(dm);
            const size_t lds = 4 * Score16Lds(vpl, dm.topk).bytes();
            const void *fn = vpl == 8 ? (const void *)select_score16_kernel<8>
                             : vpl == 4 ? (const void *)select_score16_kernel<4>
                                        : (const void *)select_score16_kernel<2>;
            if (lds > 64 * 1024) {
                const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return (int)e;
            }
            if (vpl == 8)
                hipLaunchKernelGGL(select_score16_kernel<8>, dim3((uint32_t)n_wg), dim3(256), lds, stream, dm, q, ckp,
                                   nt_cap, seqlens, lse2, R, nb_cap, n_tiles, block_idx);
            else if (vpl == 4)
                hipLaunchKernelGGL(select_score16_kernel<4>, dim3((uint32_t)n_wg), dim3(256), lds, stream, dm, q, ckp,
                                   nt_cap, seqlens, lse2, R, nb_cap, n_tiles, block_idx);
            else
                hipLaunchKernelGGL(select_score16_kernel<2>, dim3((uint32_t)n_wg), dim3(256), lds, stream, dm, q, ckp,
                                   nt_cap, seqlens, lse2, R, nb_cap, n_tiles, block_idx);
        }
        timing_end(stream);
    }
    if (!dm.shared_q || scores_out) return (int)hipGetLastError();   // ranked inside pass 2, or scores wanted
    return launch_select_pick(dm, seqlens, R, nb_cap, block_idx, stream);
}

}  // namespace infllmv2
