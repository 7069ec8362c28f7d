// Stage 2, prefill: block selection for every query token (section 2.1.2, "Dynamic Contextual
// Block Selection", Eq. 1, "Top-K Blocks Sharing", "Efficient Top-K Implementation").
//
// The relevance softmax runs over all visible semantic kernels and the group mean is taken
// AFTER it, so the scores cannot be produced by an online softmax: two passes over the
// compressed keys are needed ("Efficient Top-K Implementation").
//   pass 1  lse[token, head] = log2 sum_jh 2^(z)          z = scale*log2(e) * <q, ck_jh>
//   pass 2  r[token, jh] = (1/G) sum_head 2^(z - lse), floored at 2^-100;
//           R[token, j]  = max of r over the kernels {4j-1 .. 4j+3} that intersect block j
//   top-k   forced blocks to +inf, pick the largest, ties to the lower index.
// Both passes are causal GEMMs Q (tokens*heads x 128) . CK^T on 16x16x32 bf16 MFMA with the
// 64-kernel CK chunk staged in LDS; a wavefront keeps its query fragments in registers.
// Row tiles: 16 consecutive (token, head) rows of one key-value head, i.e. 16/G tokens.
#include "common.h"

namespace infllmv2 {

constexpr int kChunk = 64;        // semantic kernels per LDS stage (= 16 key-value blocks)
constexpr int kCkPitch = 136;     // bf16 elements per CK row in LDS (272 B)

template <int G> struct SelCfg {
    static constexpr int kTokPerTile = 16 / G;                     // tokens in one 16-row MFMA tile
    static constexpr int kTiles = (G == 1) ? 1 : (G / 2);           // row tiles per wavefront
    static constexpr int kTokPerWave = kTiles * kTokPerTile;        // 8 (16 when G == 1)
    static constexpr int kTokPerWg = 4 * kTokPerWave;
};

// Kernels visible to the query at position i: those lying wholly at or before i.
__device__ inline int n_visible(int i) { return num_kernels(i + 1); }

__device__ inline void stage_ck_chunk(__bf16 *lds, const __bf16 *ckb, int64_t st, int jh0, int n_valid,
                                      int tid) {
    const int sc = tid & 15, sr = tid >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = sr + 16 * i;
        uint4 x = {0u, 0u, 0u, 0u};
        if (jh0 + r < n_valid) x = *reinterpret_cast<const uint4 *>(ckb + (int64_t)(jh0 + r) * st + 8 * sc);
        *reinterpret_cast<uint4 *>(&lds[r * kCkPitch + 8 * sc]) = x;
    }
}

template <int G>
__device__ inline void load_q_tiles(bf16x8 (&qf)[SelCfg<G>::kTiles][4], const Tensor &q, int b, int h,
                                    int tok_wave0, int L, int n, int g) {
    using C = SelCfg<G>;
#pragma unroll
    for (int mt = 0; mt < C::kTiles; ++mt) {
        const int tok = tok_wave0 + mt * C::kTokPerTile + n / G;
        const int head = h * G + n % G;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[mt][ks] = zero8();
            if (tok < L)
                qf[mt][ks] = load8(q.ptr + b * q.sb + (int64_t)tok * q.st + (int64_t)head * q.sh + 32 * ks + 8 * g);
        }
    }
}

// ---- pass 1: log-sum-exp per (token, head) over the visible kernels -------------------------
// MFMA computes Z^T = CK . Q^T: lane = one (token, head) row, its 4 accumulator entries are 4
// consecutive kernels, so the running (max, sum) is lane-local until the final 4-group merge.
template <int G>
__global__ __launch_bounds__(256) void select_lse_kernel(Dims dm, Tensor q, Tensor ck,
                                                          const int32_t *__restrict__ seqlens,
                                                          float *__restrict__ lse2, int32_t n_tiles) {
    using C = SelCfg<G>;
    __shared__ __align__(16) __bf16 cks[kChunk * kCkPitch];
    const int tile = blockIdx.x % n_tiles;
    const int h = (blockIdx.x / n_tiles) % dm.Hkv;
    const int b = blockIdx.x / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int t0 = tile * C::kTokPerWg;
    if (t0 >= L) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int tok_wave0 = t0 + wave * C::kTokPerWave;

    bf16x8 qf[C::kTiles][4];
    load_q_tiles<G>(qf, q, b, h, tok_wave0, L, n, g);
    float m_run[C::kTiles], s_run[C::kTiles];
    int nvis[C::kTiles];
#pragma unroll
    for (int mt = 0; mt < C::kTiles; ++mt) {
        m_run[mt] = -INFINITY;
        s_run[mt] = 0.f;
        nvis[mt] = n_visible(tok_wave0 + mt * C::kTokPerTile + n / G);
    }
    const int last_tok = min(t0 + C::kTokPerWg, (int)L) - 1;
    const int nvis_wg = n_visible(last_tok);
    const int nvis_wave_min = n_visible(tok_wave0);
    const int n_valid = num_kernels(L);
    const __bf16 *ckb = ck.ptr + b * ck.sb + h * ck.sh;

    for (int jh0 = 0; jh0 < nvis_wg; jh0 += kChunk) {
        __syncthreads();
        stage_ck_chunk(cks, ckb, ck.st, jh0, n_valid, tid);
        __syncthreads();
        f32x4 z[C::kTiles][4];
#pragma unroll
        for (int mt = 0; mt < C::kTiles; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) z[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                bf16x8 a = load8(&cks[(16 * nt + n) * kCkPitch + 32 * ks + 8 * g]);
#pragma unroll
                for (int mt = 0; mt < C::kTiles; ++mt) z[mt][nt] = mfma16(a, qf[mt][ks], z[mt][nt]);
            }
        const bool edge = jh0 + kChunk > nvis_wave_min;     // some entry of this wave may be masked
#pragma unroll
        for (int mt = 0; mt < C::kTiles; ++mt) {
            float mx = -INFINITY;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float x = z[mt][nt][j] * dm.scale_log2;
                    if (edge && jh0 + 16 * nt + 4 * g + j >= nvis[mt]) x = -INFINITY;
                    z[mt][nt][j] = x;
                    mx = fmaxf(mx, x);
                }
            const float m_new = fmaxf(m_run[mt], mx);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            float acc = s_run[mt] * fast_exp2(m_run[mt] - m_use);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc += fast_exp2(z[mt][nt][j] - m_use);
            s_run[mt] = acc;
            m_run[mt] = m_new;
        }
    }
#pragma unroll
    for (int mt = 0; mt < C::kTiles; ++mt) {
        const float M = xgroup_max(m_run[mt]);
        const float m_use = M == -INFINITY ? 0.f : M;
        const float S = xgroup_sum(s_run[mt] * fast_exp2(m_run[mt] - m_use));
        const int tok = tok_wave0 + mt * C::kTokPerTile + n / G;
        if (g == 0 && tok < L)
            lse2[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + n % G] = M + fast_log2(S);
    }
}

// ---- pass 2: group-mean kernel scores, 5-wide / stride-4 max over kernels -> block scores ----
// MFMA computes Z = Q . CK^T: lane = one kernel, its 4 accumulator entries are 4 consecutive
// (token, head) rows, so the sum over a token's heads is 3 adds plus at most 2 cross-group adds.
//
// kFused: the block scores stay in LDS, a chunk of kPickChunk blocks per token; when a chunk is complete
// each wavefront merges it into the running top n_pick of its tokens (wave_topk over the chunk's scores
// plus the carried picks), and after the last chunk adds the forced blocks and writes the rows.  No
// score matrix, no separate ranking kernel.  !kFused: the scores R[token, j] go to memory (only the
// query-block-shared comparison variant, which averages them over 64 tokens first, needs that).
constexpr int kPickVpl = 4, kPickChunk = 64 * kPickVpl;           // blocks per chunk of the in-kernel top-k
template <int G> struct ScoreLds {                                 // dynamic LDS of the fused variant
    int carry_pitch, topk_words;
    __host__ __device__ explicit ScoreLds(int topk)
        : carry_pitch((topk + 1) & ~1), topk_words(64 + topk_cand_cap(topk, kPickVpl + 1)) {}
    __host__ __device__ size_t bytes() const {
        return (size_t)SelCfg<G>::kTokPerWg * kPickChunk * sizeof(float) +
               ((size_t)SelCfg<G>::kTokPerWg * carry_pitch + 4 * (size_t)topk_words) * sizeof(uint64_t);
    }
};

template <int G, bool kFused>
__global__ __launch_bounds__(256) void select_score_kernel(Dims dm, Tensor q, Tensor ck,
                                                            const int32_t *__restrict__ seqlens,
                                                            const float *__restrict__ lse2,
                                                            float *__restrict__ R, int32_t nb_cap,
                                                            int32_t n_tiles, int32_t *__restrict__ block_idx) {
    using C = SelCfg<G>;
    constexpr int TL = (G >= 4) ? 1 : 4 / G;     // tokens held by one lane of a row tile
    constexpr int RL = (G >= 4) ? 4 : G;         // rows of one token held by one lane
    __shared__ __align__(16) __bf16 cks[kChunk * kCkPitch];
    __shared__ float rs[C::kTokPerWg][kChunk + 2];   // slot 0: kernel jh0-1 (halo), slot 1+x: jh0+x
    extern __shared__ __align__(16) unsigned char score_smem[];
    const ScoreLds<G> lay(dm.topk);
    float *Rl = reinterpret_cast<float *>(score_smem);                                   // [kTokPerWg][kPickChunk]
    uint64_t *carry = reinterpret_cast<uint64_t *>(Rl + C::kTokPerWg * kPickChunk);      // [kTokPerWg][carry_pitch]
    const int tile = blockIdx.x % n_tiles;
    const int h = (blockIdx.x / n_tiles) % dm.Hkv;
    const int b = blockIdx.x / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int t0 = tile * C::kTokPerWg;
    if (t0 >= L) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int tok_wave0 = t0 + wave * C::kTokPerWave;

    bf16x8 qf[C::kTiles][4];
    load_q_tiles<G>(qf, q, b, h, tok_wave0, L, n, g);
    // lane holds rows 4g+j of each row tile: their log-sum-exps
    float lse_r[C::kTiles][4];
#pragma unroll
    for (int mt = 0; mt < C::kTiles; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = 4 * g + j;
            const int tok = tok_wave0 + mt * C::kTokPerTile + r / G;
            lse_r[mt][j] = tok < L ? lse2[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + r % G] : 0.f;
        }
    const int last_tok = min(t0 + C::kTokPerWg, (int)L) - 1;
    const int nvis_wg = n_visible(last_tok);
    const int n_valid = num_kernels(L);
    const __bf16 *ckb = ck.ptr + b * ck.sb + h * ck.sh;
    for (int i = tid; i < C::kTokPerWg; i += 256) rs[i][0] = -INFINITY;
    // the tokens of a workgroup share their own block (kTokPerWg divides 64), hence the candidate range
    const int b_own = t0 / kBlock, n_blk = b_own + 1;
    const int n_sel = dm.topk < n_blk ? dm.topk : n_blk;
    const int n_init = dm.n_init < n_blk ? dm.n_init : n_blk;                 // forced leading blocks
    const int lo_local = max(n_init, b_own - dm.n_local + 1);                 // forced trailing: lo_local..b_own
    const int jc_max = lo_local - 1;                                          // candidates: n_init..jc_max
    const int n_pick = max(0, n_sel - (n_init + (b_own - lo_local + 1)));
    uint64_t *tk_lds = carry + C::kTokPerWg * lay.carry_pitch + wave * lay.topk_words;
    if (kFused)
        for (int i = tid; i < C::kTokPerWg * lay.carry_pitch; i += 256) carry[i] = 0ull;
    // merges the chunk of blocks j0 .. j0 + kPickChunk - 1 into the running picks of this wavefront's tokens
    auto merge_chunk = [&](int j0) {
        for (int u = 0; u < C::kTokPerWave; ++u) {
            const int tloc = wave * C::kTokPerWave + u;
            if (t0 + tloc >= L || n_pick <= 0) break;
            uint64_t el[kPickVpl + 1];
#pragma unroll
            for (int s2 = 0; s2 < kPickVpl; ++s2)
                el[s2] = pick_element(Rl[tloc * kPickChunk + lane + 64 * s2], j0 + lane + 64 * s2, n_init, jc_max);
            el[kPickVpl] = lane < n_pick ? carry[tloc * lay.carry_pitch + lane] : 0ull;
            const uint64_t res = wave_topk<kPickVpl + 1>(el, n_pick, tk_lds, lane);
            if (lane < n_pick) carry[tloc * lay.carry_pitch + lane] = res;
        }
    };

    for (int jh0 = 0; jh0 < nvis_wg; jh0 += kChunk) {
        __syncthreads();
        stage_ck_chunk(cks, ckb, ck.st, jh0, n_valid, tid);
        __syncthreads();
        f32x4 z[C::kTiles][4];
#pragma unroll
        for (int mt = 0; mt < C::kTiles; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) z[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                bf16x8 bq = load8(&cks[(16 * nt + n) * kCkPitch + 32 * ks + 8 * g]);
#pragma unroll
                for (int mt = 0; mt < C::kTiles; ++mt) z[mt][nt] = mfma16(qf[mt][ks], bq, z[mt][nt]);
            }
#pragma unroll
        for (int mt = 0; mt < C::kTiles; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                float e[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) e[j] = fast_exp2(z[mt][nt][j] * dm.scale_log2 - lse_r[mt][j]);
                const int jh = jh0 + 16 * nt + n;
#pragma unroll
                for (int tl = 0; tl < TL; ++tl) {
                    float vsum = 0.f;
#pragma unroll
                    for (int jj = 0; jj < RL; ++jj) vsum += e[tl * RL + jj];
                    if (G >= 8) vsum += __shfl_xor(vsum, 16);
                    if (G >= 16) vsum += __shfl_xor(vsum, 32);
                    // token of rows 4g + tl*RL ..: local index inside the workgroup's tile
                    const int tloc = wave * C::kTokPerWave + mt * C::kTokPerTile + (4 * g + tl * RL) / G;
                    const bool writer = ((4 * g + tl * RL) % G) == 0;
                    if (writer) {
                        float r = fminf(fmaxf(vsum * (1.f / G), kScoreFloor), kScoreCeil);
                        if (jh >= n_visible(t0 + tloc)) r = -INFINITY;
                        rs[tloc][1 + 16 * nt + n] = r;
                    }
                }
            }
        __syncthreads();
        // block scores of blocks jh0/4 .. jh0/4+15: kernels 4j-1 .. 4j+3 -> slots 4jb .. 4jb+4
        for (int i = tid; i < C::kTokPerWg * 16; i += 256) {
            const int tloc = i >> 4, jb = i & 15;
            const int tok = t0 + tloc, j = (jh0 >> 2) + jb;
            if (tok < L && j <= tok / kBlock) {
                float r = rs[tloc][4 * jb];
#pragma unroll
                for (int x = 1; x < 5; ++x) r = fmaxf(r, rs[tloc][4 * jb + x]);
                if (kFused) Rl[tloc * kPickChunk + (j & (kPickChunk - 1))] = r;
                else R[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * nb_cap + j] = r;
            }
        }
        __syncthreads();
        for (int i = tid; i < C::kTokPerWg; i += 256) rs[i][0] = rs[i][kChunk];
        // a chunk of blocks is complete (the barrier that opens the next stage orders the merge before
        // the next chunk's scores)
        if (kFused && (((jh0 >> 2) + 16) & (kPickChunk - 1)) == 0) merge_chunk((jh0 >> 2) + 16 - kPickChunk);
    }
    // Blocks past the last scored chunk (only the last ones of a token can be).  Of their kernels only
    // the left neighbour of the first one, 4*j_done - 1 = the last kernel of the last chunk, can be
    // visible: its score sits in the halo slot.  It decides when the token's own block is a candidate
    // (no forced local blocks).
    __syncthreads();
    const int j_done = ((nvis_wg + kChunk - 1) / kChunk) * 16;
    for (int i = tid; i < C::kTokPerWg * 4; i += 256) {
        const int tloc = i >> 2, tok = t0 + tloc, j = j_done + (i & 3);
        if (tok < L && j <= tok / kBlock) {
            const float r = (i & 3) == 0 ? rs[tloc][0] : -INFINITY;
            if (kFused) Rl[tloc * kPickChunk + (j & (kPickChunk - 1))] = r;
            else R[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * nb_cap + j] = r;
        }
    }
    if (kFused) {
        __syncthreads();
        merge_chunk(j_done & ~(kPickChunk - 1));             // the last, partial chunk: it holds block j_done
        for (int u = 0; u < C::kTokPerWave; ++u) {
            const int tloc = wave * C::kTokPerWave + u;
            if (t0 + tloc >= L) break;
            const int picked = lane < n_pick ? (int)~(uint32_t)carry[tloc * lay.carry_pitch + lane] : 0;
            write_block_row(picked, n_pick, n_sel, n_init, lo_local, dm.topk,
                            block_idx + (((int64_t)b * dm.Hkv + h) * dm.max_seqlen + t0 + tloc) * dm.topk, lane);
        }
    }
}

// ---- top-k over stored block scores: one wavefront per row ---------------------------------------
// Only the query-block-shared comparison variant still ranks a stored score matrix (its rows are
// averages over 64 tokens); the method itself ranks inside pass 2.  Candidates are the blocks
// n_init .. b_own - n_local; the forced ones are added afterwards.  Scores are positive floats, so
// their bit patterns order like unsigned integers.  An element is the 64-bit word  key << 32 | ~block
// with key = bits of the score (1 for a block without visible kernel, -inf): larger word = better
// element, ties go to the lower block index, no two elements are equal; words below 2^32 are "not a
// candidate".  Lane l keeps blocks l, l+64, ... in registers; wave_topk ranks them.
constexpr int kPickRowsPerWg = 4;

template <int VPL>
__global__ __launch_bounds__(256) void select_pick_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                           const float *__restrict__ R, int32_t nb_cap,
                                                           int32_t *__restrict__ block_idx, int32_t row_tokens) {
    extern __shared__ __align__(16) unsigned char pick_smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t *lds = reinterpret_cast<uint64_t *>(pick_smem) + (size_t)wave * (64 + topk_cand_cap(dm.topk, VPL));
    // a row is one query token, or (row_tokens = 64, the query-block-shared variant) one query block,
    // which selects like its last token
    const int rows_per_seq = (dm.max_seqlen + row_tokens - 1) / row_tokens;
    const int64_t row = (int64_t)blockIdx.x * kPickRowsPerWg + wave;
    const int64_t rows = (int64_t)dm.batch * dm.Hkv * rows_per_seq;
    if (row >= rows) return;
    const int b = row / ((int64_t)rows_per_seq * dm.Hkv);
    const float *Rr = R + row * nb_cap;
    float r[VPL];                                                             // every load issued before any use
#pragma unroll
    for (int s = 0; s < VPL; ++s) r[s] = Rr[min(lane + 64 * s, nb_cap - 1)];
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int tok0 = (int)(row % rows_per_seq) * row_tokens;
    if (tok0 >= L) return;
    const int tok = min(tok0 + row_tokens - 1, L - 1);
    const int b_own = tok / kBlock, n_blk = b_own + 1;
    const int n_sel = dm.topk < n_blk ? dm.topk : n_blk;
    const int n_init = dm.n_init < n_blk ? dm.n_init : n_blk;                 // forced leading blocks
    const int lo_local = max(n_init, b_own - dm.n_local + 1);                 // forced trailing: lo_local..b_own
    const int jc_max = lo_local - 1;                                          // candidates: n_init..jc_max
    const int n_pick = n_sel - (n_init + (b_own - lo_local + 1));
    int picked = 0;
    if (n_pick > 0) {                                                         // uniform over the wavefront
        uint64_t el[VPL];
#pragma unroll
        for (int s = 0; s < VPL; ++s) el[s] = pick_element(r[s], lane + 64 * s, n_init, jc_max);
        picked = (int)~(uint32_t)wave_topk<VPL>(el, n_pick, lds, lane);
    }
    write_block_row(picked, n_pick, n_sel, n_init, lo_local, dm.topk, block_idx + row * dm.topk, lane);
}

// Fallback for rows longer than 64*32 blocks: scans the row in memory once per pick.
__global__ __launch_bounds__(256) void select_pick_scan_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                                const float *__restrict__ R, int32_t nb_cap,
                                                                int32_t *__restrict__ block_idx, int32_t row_tokens) {
    const int lane = threadIdx.x & 63;
    const int rows_per_seq = (dm.max_seqlen + row_tokens - 1) / row_tokens;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t rows = (int64_t)dm.batch * dm.Hkv * rows_per_seq;
    if (row >= rows) return;
    const int b = row / ((int64_t)rows_per_seq * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int tok0 = (int)(row % rows_per_seq) * row_tokens;
    if (tok0 >= L) return;
    const int tok = min(tok0 + row_tokens - 1, L - 1);
    const int b_own = tok / kBlock, n_blk = b_own + 1;
    const int n_sel = dm.topk < n_blk ? dm.topk : n_blk;
    const float *Rr = R + row * nb_cap;
    float last_s = INFINITY;
    int last_j = -1;
    int mine = 0x7fffffff;
    for (int c = 0; c < n_sel; ++c) {
        float best_s = -INFINITY;
        int best_j = 0x7fffffff;
        for (int j = lane; j < n_blk; j += 64) {
            float sc = (j < dm.n_init || j > b_own - dm.n_local) ? INFINITY : Rr[j];
            const bool after = sc < last_s || (sc == last_s && j > last_j);
            if (after && (sc > best_s || (sc == best_s && j < best_j))) {
                best_s = sc;
                best_j = j;
            }
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const float os = __shfl_xor(best_s, o);
            const int oj = __shfl_xor(best_j, o);
            if (os > best_s || (os == best_s && oj < best_j)) {
                best_s = os;
                best_j = oj;
            }
        }
        last_s = best_s;
        last_j = best_j;
        if (lane == c) mine = best_j;
    }
    int rank = 0;
    for (int c = 0; c < n_sel; ++c) rank += __shfl(mine, c) < mine ? 1 : 0;
    int32_t *o = block_idx + row * dm.topk;
    if (lane < n_sel) o[rank] = mine;
    else if (lane < dm.topk) o[lane] = -1;
}

int32_t select_scores_pitch(const Dims &dm) {
    return (int32_t)(((size_t)(dm.max_seqlen + kBlock - 1) / kBlock + 15) / 16 * 16);
}
size_t select_scores_bytes(const Dims &dm) {            // only the query-block-shared variant stores scores
    if (!dm.shared_q) return 0;
    return (size_t)dm.batch * dm.Hkv * dm.max_seqlen * select_scores_pitch(dm) * sizeof(float);
}
size_t select_shared_scores_bytes(const Dims &dm) {     // per-query-block scores of the shared variant, behind the per-token ones
    if (!dm.shared_q) return 0;
    return (size_t)dm.batch * dm.Hkv * ((dm.max_seqlen + kBlock - 1) / kBlock) * select_scores_pitch(dm) * sizeof(float);
}

// Query-block-shared variant (not the report's method; section 2.1.3 argues for token-level queries):
// the block scores of the 64 tokens of a query block are averaged, one row per query block.
// grid (n_qb, Hkv, B), 256 threads over the candidate blocks.
__global__ __launch_bounds__(256) void reduce_scores_kernel(Dims dm, const int32_t *__restrict__ seqlens,
                                                             const float *__restrict__ R, int32_t nb_cap,
                                                             float *__restrict__ Rq, int32_t n_qb) {
    const int I = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int t0 = I * kBlock, n_tok = min(kBlock, L - t0);
    if (n_tok <= 0) return;
    const int64_t bh = (int64_t)b * dm.Hkv + h;
    const int j_hi = I - dm.n_local;                      // candidates n_init .. I - n_local: wholly visible to every token
    for (int j = dm.n_init + threadIdx.x; j <= j_hi; j += 256) {
        float acc = 0.f;
        for (int t = 0; t < n_tok; ++t) acc += R[(bh * dm.max_seqlen + t0 + t) * nb_cap + j];
        Rq[(bh * n_qb + I) * nb_cap + j] = acc / (float)n_tok;
    }
}

int launch_select_pick(const Dims &dm, const int32_t *seqlens, const float *R, int32_t nb_cap,
                       int32_t *block_idx, hipStream_t stream) {
    int32_t row_tokens = 1;
    if (dm.shared_q) {                                    // average over the query blocks first; Rq sits behind R
        const int32_t n_qb = (dm.max_seqlen + kBlock - 1) / kBlock;
        if (n_qb <= 0 || dm.batch <= 0) return 0;
        float *Rq = const_cast<float *>(R) + select_scores_bytes(dm) / sizeof(float);
        timing_begin("reduce_scores_kernel", stream);
        hipLaunchKernelGGL(reduce_scores_kernel, dim3(n_qb, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, seqlens, R,
                           nb_cap, Rq, n_qb);
        timing_end(stream);
        R = Rq;
        row_tokens = kBlock;
    }
    const int rows_per_seq = (dm.max_seqlen + row_tokens - 1) / row_tokens;
    const int64_t rows = (int64_t)dm.batch * dm.Hkv * rows_per_seq;
    if (rows <= 0) return 0;
    const dim3 grid((uint32_t)((rows + 3) / 4));
    const int n_blocks = (dm.max_seqlen + kBlock - 1) / kBlock;
    const int vpl = n_blocks <= 64 * 4 ? 4 : n_blocks <= 64 * 8 ? 8 : n_blocks <= 64 * 16 ? 16 : 32;
    const size_t lds = (size_t)kPickRowsPerWg * (64 + topk_cand_cap(dm.topk, vpl)) * sizeof(uint64_t);
    timing_begin("select_pick_kernel", stream);
    if (n_blocks > 64 * 32 || lds > 64 * 1024)           // very long rows or very wide top-k: generic scan
        hipLaunchKernelGGL(select_pick_scan_kernel, grid, dim3(256), 0, stream, dm, seqlens, R, nb_cap, block_idx, row_tokens);
    else if (vpl == 4)
        hipLaunchKernelGGL((select_pick_kernel<4>), grid, dim3(256), lds, stream, dm, seqlens, R, nb_cap, block_idx, row_tokens);
    else if (vpl == 8)
        hipLaunchKernelGGL((select_pick_kernel<8>), grid, dim3(256), lds, stream, dm, seqlens, R, nb_cap, block_idx, row_tokens);
    else if (vpl == 16)
        hipLaunchKernelGGL((select_pick_kernel<16>), grid, dim3(256), lds, stream, dm, seqlens, R, nb_cap, block_idx, row_tokens);
    else
        hipLaunchKernelGGL((select_pick_kernel<32>), grid, dim3(256), lds, stream, dm, seqlens, R, nb_cap, block_idx, row_tokens);
    timing_end(stream);
    return (int)hipGetLastError();
}

size_t select_prefill_ws_bytes(const Dims &dm) {
    if (dm.G == 16) return select_prefill16_ws_bytes(dm);
    size_t lse = (size_t)dm.batch * dm.max_seqlen * dm.Hq * sizeof(float);
    lse = (lse + 255) / 256 * 256;
    return lse + select_scores_bytes(dm) + select_shared_scores_bytes(dm);
}

template <int G>
static int launch_select_prefill_g(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                                   int32_t *block_idx, void *ws, hipStream_t stream, float *scores_out,
                                   int32_t scores_pitch) {
    using C = SelCfg<G>;
    const int32_t nb_cap = scores_out ? scores_pitch : select_scores_pitch(dm);
    size_t lse_bytes = (size_t)dm.batch * dm.max_seqlen * dm.Hq * sizeof(float);
    lse_bytes = (lse_bytes + 255) / 256 * 256;
    float *lse2 = reinterpret_cast<float *>(ws);
    float *R = scores_out ? scores_out : reinterpret_cast<float *>(reinterpret_cast<char *>(ws) + lse_bytes);
    const int32_t n_tiles = (dm.max_seqlen + C::kTokPerWg - 1) / C::kTokPerWg;
    const int64_t n_wg = (int64_t)n_tiles * dm.Hkv * dm.batch;
    if (n_wg <= 0) return 0;
    timing_begin("select_lse_kernel", stream);
    hipLaunchKernelGGL(select_lse_kernel<G>, dim3((uint32_t)n_wg), dim3(256), 0, stream, dm, q, ck,
                       seqlens, lse2, n_tiles);
    timing_end(stream);
    timing_begin("select_score_kernel", stream);
    if (dm.shared_q || scores_out) {
        hipLaunchKernelGGL((select_score_kernel<G, false>), dim3((uint32_t)n_wg), dim3(256), 0, stream, dm, q, ck,
                           seqlens, lse2, R, nb_cap, n_tiles, block_idx);
        timing_end(stream);
        if (scores_out) return (int)hipGetLastError();    // the caller wanted the scores, not the block sets
        return launch_select_pick(dm, seqlens, R, nb_cap, block_idx, stream);
    }
    const size_t lds = ScoreLds<G>(dm.topk).bytes();     // beside 26 to 34 KiB of static LDS
    const hipError_t e = hipFuncSetAttribute((const void *)select_score_kernel<G, true>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return (int)e;
    hipLaunchKernelGGL((select_score_kernel<G, true>), dim3((uint32_t)n_wg), dim3(256), lds, stream, dm, q, ck,
                       seqlens, lse2, R, nb_cap, n_tiles, block_idx);
    timing_end(stream);
    return (int)hipGetLastError();
}

// scores_out != null: stop after pass 2 and leave the block scores of the candidate blocks in
// scores_out[((b * Hkv + h) * max_seqlen + t) * scores_pitch + j] instead of ranking them.
int launch_select_prefill(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                          int32_t *block_idx, void *ws, hipStream_t stream, float *scores_out,
                          int32_t scores_pitch) {
    switch (dm.G) {
        case 1: return launch_select_prefill_g<1>(dm, q, ck, seqlens, block_idx, ws, stream, scores_out, scores_pitch);
        case 2: return launch_select_prefill_g<2>(dm, q, ck, seqlens, block_idx, ws, stream, scores_out, scores_pitch);
        case 4: return launch_select_prefill_g<4>(dm, q, ck, seqlens, block_idx, ws, stream, scores_out, scores_pitch);
        case 8: return launch_select_prefill_g<8>(dm, q, ck, seqlens, block_idx, ws, stream, scores_out, scores_pitch);
        case 16: return launch_select_prefill16(dm, q, ck, seqlens, block_idx, ws, stream, scores_out, scores_pitch);
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace infllmv2
