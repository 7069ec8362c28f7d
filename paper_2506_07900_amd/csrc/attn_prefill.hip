// Stage 3, prefill: exact softmax attention of every query token over its own selected
// key-value blocks (section 2.1.1, second stage; section 2.1.3 "Different Granularity for
// Query and Key-Value Tokens": the query unit is a token, the key-value unit a 64-token block).
//
// Two kernels.
//
// pack_kv_kernel re-lays every 64-token block of the K and V caches into "fragment-major" order
// in the workspace: the 16 bytes a lane feeds to one 16x16x32 MFMA are contiguous and the 64
// lanes of a fragment are consecutive, so a wavefront fetches an operand fragment as one fully
// coalesced 1 KiB read straight into registers.  V is transposed on the way (the value product
// contracts over keys, which are the strided axis of the cache).
//
// attn_prefill_kernel: a wavefront owns kTok consecutive query tokens of one key-value head and
// works alone -- no LDS, no barriers.  The G (<=16) query heads of a token fill the 16 columns of
// one MFMA tile, so per-token block sets cost no padded matrix work when G = 16.  The wavefront
// walks the union of its tokens' block lists in ascending order; each fragment it loads is used
// for every one of its tokens that selected the block.  Both contractions are computed
// transposed so that no register shuffles are needed:
//   S^T[key, head] = K[key, :] . Q[head, :]            A = K fragment,   B = Q (registers)
//   O^T[c,  head] += V^T[c, key] . P^T[key, head]       A = V^T fragment, B = P^T taken straight
// from the accumulator layout of S^T (lane = head column, 4 consecutive keys per 16-lane group),
// with the key order inside the packed V^T rows permuted to match.
#include "common.h"

namespace infllmv2 {

constexpr int kFragsPerOperand = 16;                     // 16 fragments of 1 KiB = one 16 KiB operand block
constexpr int kPackedBlockU4 = 2 * kFragsPerOperand * 64; // uint4 per packed (K, V) block: 32 KiB

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

// ---- re-layout of one 64-token block per workgroup -------------------------------------------------
// K fragment (ks, mt), lane (g, m):  K[64j + 16mt + m][32ks + 8g .. +7]
// V fragment (dt, kk), lane (g, m), element e:  V[64j + 32kk + (e<4 ? 4g+e : 16+4g+e-4)][16dt + m]
__global__ __launch_bounds__(256) void pack_kv_kernel(Dims dm, Tensor k, Tensor v,
                                                       const int32_t *__restrict__ seqlens,
                                                       uint4 *__restrict__ kvp, int32_t nb_cap) {
    __shared__ __align__(16) __bf16 Ks[kBlock * 136];
    __shared__ __align__(16) __bf16 Vs[kBlock * 136];
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
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
    uint4 *dst = kvp + ((((int64_t)b * dm.Hkv + h) * nb_cap + j) * kPackedBlockU4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;                 // K chunk: fragment f = c/64, lane = c%64
        const int f = c >> 6, lane = c & 63, m = lane & 15, g = lane >> 4;
        const int ks = f >> 2, mt = f & 3;
        dst[c] = *reinterpret_cast<const uint4 *>(&Ks[(16 * mt + m) * 136 + 32 * ks + 8 * g]);
    }
    const uint16_t *Vu = reinterpret_cast<const uint16_t *>(Vs);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;                 // V chunk
        const int f = c >> 6, lane = c & 63, m = lane & 15, g = lane >> 4;
        const int dt = f >> 1, kk = f & 1;
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const int e = 2 * e2;                    // elements e, e+1 are consecutive keys
            const int key = 32 * kk + (e < 4 ? 4 * g + e : 16 + 4 * g + e - 4);
            const uint32_t lo = Vu[key * 136 + 16 * dt + m];
            const uint32_t hi = Vu[(key + 1) * 136 + 16 * dt + m];
            w[e2] = lo | (hi << 16);
        }
        dst[kFragsPerOperand * 64 + c] = uint4{w[0], w[1], w[2], w[3]};
    }
}

// ---- attention ---------------------------------------------------------------------------------------
// A block is processed as two halves of 32 keys.  The operand fragments of a block are fetched in
// 8 units of 4 fragments (4 KiB per wavefront), in the order they are consumed:
//   half hs:  K rows of key tile 2hs (all four 32-channel k-steps), K rows of key tile 2hs+1,
//             V^T of the half's 32 keys for channel tiles 0..3, then for channel tiles 4..7
// They rotate through a ring of kNU register buffers: as soon as the matrix cores have consumed
// a unit, the load of the unit kNU places further down the stream (same block, or the next block
// of the wavefront's list) is issued into the same registers, so loads stay in flight under the
// wavefront's own arithmetic.
//
// The softmax keeps a per-head reference exponent taken from the data and re-bases it only when
// a partial sum leaves the safe range (or on first use, when it is still NaN): the common path is
// one fma, one exp2 and one add per probability, with no running maximum.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr float kPsumLimit = 0x1p40f;
constexpr int kNone = 0x7fffffff;
constexpr int kBlkBits = 27, kBlkMask = (1 << kBlkBits) - 1;

// probabilities 2^(s*c + ne) of 32 keys (two key tiles) of one token in MFMA B layout, and their sum
__device__ __forceinline__ float half_probs(const f32x4 (&s)[2], float c, float ne, bf16x8 &p8) {
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p = fast_exp2(__builtin_fmaf(s[t][j], c, ne));
            sum += p;
            p8[4 * t + j] = (__bf16)p;
        }
    return sum;
}

template <int kTok, int kNU, int kWavesPerSimd>
__global__ __launch_bounds__(256, kWavesPerSimd) void attn_prefill_kernel(Dims dm, Tensor q, const uint4 *__restrict__ kvp,
                                                            int32_t nb_cap,
                                                            const int32_t *__restrict__ seqlens,
                                                            const int32_t *__restrict__ block_idx,
                                                            Tensor out, float *__restrict__ lse,
                                                            int32_t n_tiles) {
    static_assert(kNU == 4 || kNU == 8, "ring of 4 or 8 units");
    static_assert(kTok <= 4 && 64 % kTok == 0, "membership bits / one own block per wavefront");
    // a workgroup is 4 independent wavefronts covering 4*kTok consecutive tokens
    const uint32_t vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int tile = vid % n_tiles;
    const int h = (vid / n_tiles) % dm.Hkv;
    const int b = vid / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = (tile * 4 + wave) * kTok;             // this wavefront's first token
    if (t0 >= L) return;
    const int b_own = t0 / kBlock;                       // kTok divides 64: one own block per wavefront
    const int n = lane & 15, g = lane >> 4;              // MFMA column (query head) and 16-lane group
    const int G = dm.G;
    const float c = dm.scale_log2;

    bf16x8 qf[kTok][4];
    f32x4 o[kTok][8];
    float neg_m[kTok], l_run[kTok];
    int own[kTok];                                       // lane e < topk holds entry e of the block list
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const int tok = t0 + u;
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
        neg_m[u] = __builtin_nanf("");
        l_run[u] = 0.f;
        int e = kNone;
        if (live && lane < dm.topk) {
            int x = block_idx[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * dm.topk + lane];
            if (x >= 0 && x <= b_own) e = x;
        }
        own[u] = e;
    }

    // Ascending union of the tokens' block lists, by counting instead of sorting: an entry's place
    // is the number of distinct smaller entries.  A token's own list holds no duplicates, so an
    // entry is a duplicate exactly when a lower-numbered token of the wavefront lists the same
    // block.  Entry i of the union ends up in lane i%64 of ul[i/64] as block | member bits << 27.
    // (A caller's row that lists a block twice, against the contract, is attended once: the copy in the
    // higher lane counts as a duplicate too, so every rank below is taken by exactly one entry.)
    int w[kTok];                                         // own[u] with duplicates removed
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        bool dup = false;
        for (int j = 0; j < dm.topk; ++j) dup |= j < lane && __builtin_amdgcn_readlane(own[u], j) == own[u];
#pragma unroll
        for (int u2 = 0; u2 < u; ++u2)
            for (int j = 0; j < dm.topk; ++j) dup |= __builtin_amdgcn_readlane(own[u2], j) == own[u];
        w[u] = dup ? kNone : own[u];
    }
    int rank[kTok], bits[kTok];
#pragma unroll
    for (int u = 0; u < kTok; ++u) rank[u] = bits[u] = 0;
#pragma unroll
    for (int u2 = 0; u2 < kTok; ++u2)
        for (int j = 0; j < dm.topk; ++j) {
            const int wj = __builtin_amdgcn_readlane(w[u2], j), xj = __builtin_amdgcn_readlane(own[u2], j);
#pragma unroll
            for (int u = 0; u < kTok; ++u) {
                rank[u] += wj < w[u] ? 1 : 0;            // kNone (absent or duplicate) is never smaller
                bits[u] |= xj == w[u] ? 1 << u2 : 0;
            }
        }
    __shared__ int ulist[4][64 * kTok];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const bool have = w[u] != kNone;
        if (have) ulist[wave][rank[u]] = w[u] | (bits[u] << kBlkBits);
        cnt += __popcll(__ballot(have));
    }
    int ul[kTok];
#pragma unroll
    for (int r = 0; r < kTok; ++r) ul[r] = ulist[wave][64 * r + lane];   // same wavefront: LDS keeps the order
    auto union_entry = [&](int i) __attribute__((always_inline)) {
        int e = __builtin_amdgcn_readlane(ul[0], i & 63);
#pragma unroll
        for (int r = 1; r < kTok; ++r)
            if ((i >> 6) == r) e = __builtin_amdgcn_readlane(ul[r], i & 63);
        return e;
    };

    const u32x4 *kv_lane = reinterpret_cast<const u32x4 *>(kvp) +
                           ((int64_t)b * dm.Hkv + h) * nb_cap * kPackedBlockU4 + lane;
    u32x4 ring[kNU][4];
    auto issue = [&](int unit, const u32x4 *bp) __attribute__((always_inline)) {
        const int hs = unit >> 2, r = unit & 3;
        if (r < 2) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) ring[unit % kNU][ks] = bp[(ks * 4 + 2 * hs + r) * 64];
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                ring[unit % kNU][i] = bp[(kFragsPerOperand + (4 * (r - 2) + i) * 2 + hs) * 64];
        }
    };

    // softmax of one member token on 32 keys: pf = P^T in bf16; re-bases the reference when needed
    auto softmax = [&](f32x4 (&s)[2], int u, bf16x8 &pf) __attribute__((always_inline)) {
        float ps = half_probs(s, c, neg_m[u], pf);
        if (__any(!(ps <= kPsumLimit))) {                 // rare: too large, inf, or NaN (no reference yet)
            float tmax = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) tmax = fmaxf(tmax, s[t][j]);
            tmax = xgroup_max(tmax) * c;                  // per head, same in the four lane groups
            const float old = neg_m[u];                   // NaN = no reference yet
            const float m_new = (old != old) ? tmax : fmaxf(-old, tmax);
            if (m_new > -INFINITY) {
                const float f = (old != old) ? 0.f : fast_exp2(-old - m_new);
                l_run[u] *= f;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[u][dt] *= f;
                neg_m[u] = -m_new;
                ps = half_probs(s, c, -m_new, pf);
            } else {                                      // every key of this head masked so far
                ps = 0.f;
                pf = zero8();
            }
        }
        l_run[u] += ps;
    };

    // Everything loaded so far (queries, block lists) has to land before the ring starts: the
    // compiler's wait-count bookkeeping otherwise merges those pending loads into the loop and
    // waits for ALL outstanding loads at the top of every iteration, which defeats the ring.
    __builtin_amdgcn_s_waitcnt(0);
    if (cnt > 0) {
        const u32x4 *bp = kv_lane + (int64_t)(union_entry(0) & kBlkMask) * kPackedBlockU4;
#pragma unroll
        for (int unit = 0; unit < kNU; ++unit) issue(unit, bp);
    }
    for (int ci = 0; ci < cnt; ++ci) {
        const int e = union_entry(ci);
        const int blk = e & kBlkMask, bits = e >> kBlkBits;
        const bool has_next = ci + 1 < cnt;
        const int en = union_entry(has_next ? ci + 1 : ci);
        const u32x4 *bp = kv_lane + (int64_t)blk * kPackedBlockU4;
        const u32x4 *bn = kv_lane + (int64_t)(en & kBlkMask) * kPackedBlockU4;
        const int key0 = blk * kBlock;
        const bool edge = (blk == b_own) || (key0 + kBlock > L);
#pragma unroll
        for (int hs = 0; hs < 2; ++hs) {
            // ---- S^T = K . Q^T for 32 keys, one key tile per unit ------------------------------
            f32x4 s[kTok][2];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int unit = 4 * hs + r;
#pragma unroll
                for (int u = 0; u < kTok; ++u) {
                    if (!((bits >> u) & 1)) continue;
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc = mfma16(__builtin_bit_cast(bf16x8, ring[unit % kNU][ks]), qf[u][ks], acc);
                    s[u][r] = acc;
                }
                if (unit + kNU < 8) issue(unit + kNU, bp);
                else issue(unit + kNU - 8, bn);      // (a harmless re-read of this block at the tail)
            }
            // ---- probabilities, P^T packed to bf16 in MFMA B layout ---------------------------
            bf16x8 pf[kTok];
#pragma unroll
            for (int u = 0; u < kTok; ++u) {
                if (!((bits >> u) & 1)) continue;
                if (edge) {
                    const int tok = t0 + u;
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (key0 + 32 * hs + 16 * t + 4 * g + j > tok) s[u][t][j] = -INFINITY;
                }
                softmax(s[u], u, pf[u]);
            }
            // ---- O^T += V^T . P^T, four channel tiles per unit --------------------------------
#pragma unroll
            for (int r = 2; r < 4; ++r) {
                const int unit = 4 * hs + r, dh = r - 2;
#pragma unroll
                for (int u = 0; u < kTok; ++u) {
                    if (!((bits >> u) & 1)) continue;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        o[u][4 * dh + i] =
                            mfma16(__builtin_bit_cast(bf16x8, ring[unit % kNU][i]), pf[u], o[u][4 * dh + i]);
                }
                if (unit + kNU < 8) issue(unit + kNU, bp);
                else issue(unit + kNU - 8, bn);      // (a harmless re-read of this block at the tail)
            }
        }
    }

    // ---- normalise and write: lane holds channels 16*dt + 4*g .. +3 of head n ------------------
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const int tok = t0 + u;
        if (tok >= L || n >= G) continue;
        const float l_tot = xgroup_sum(l_run[u]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        __bf16 *op = out.ptr + b * out.sb + (int64_t)tok * out.st + (int64_t)(h * G + n) * out.sh + 4 * g;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            bf16x4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = (__bf16)(o[u][dt][j] * inv);
            *reinterpret_cast<uint2 *>(op + 16 * dt) = __builtin_bit_cast(uint2, r);
        }
        if (g == 0)
            lse[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + n] =
                l_tot > 0.f ? (fast_log2(l_tot) - neg_m[u]) * kLn2 : -INFINITY;
    }
}

// ---- attention with one block set per query block (comparison variant) ------------------------------------
// Not the report's method (section 2.1.3: token-level queries); it shows what the same arithmetic
// reaches when the 64 tokens of a query block attend one common block list.  A workgroup takes 8
// consecutive tokens of a query block (a wavefront 2, as above) and walks the shared list in step:
// every packed block is fetched once per workgroup -- each thread carries 1/256 of the next block in
// registers while the current one is consumed -- and all four wavefronts read their operand
// fragments from LDS, which delivers several times what the L2 path does.  Only the query block's
// own key-value block needs the causal mask.
constexpr int kShTok = 2;                                // tokens per wavefront
__global__ __launch_bounds__(256, 2) void attn_prefill_shared_kernel(Dims dm, Tensor q, const uint4 *__restrict__ kvp,
                                                                      int32_t nb_cap, const int32_t *__restrict__ seqlens,
                                                                      const int32_t *__restrict__ block_idx,
                                                                      Tensor out, float *__restrict__ lse,
                                                                      int32_t n_tiles) {
    __shared__ __align__(16) u32x4 stage[2][kPackedBlockU4];
    const uint32_t vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int tile = vid % n_tiles;                      // 8 tokens
    const int h = (vid / n_tiles) % dm.Hkv;
    const int b = vid / (n_tiles * dm.Hkv);
    int32_t L = seqlens[b];
    L = L < 0 ? 0 : (L > dm.max_seqlen ? dm.max_seqlen : L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tile * 8 >= L) return;                           // uniform over the workgroup
    const int t0 = tile * 8 + wave * kShTok;             // this wavefront's first token (may lie past the end)
    const int I = (tile * 8) / kBlock;                   // the query block, and its own key-value block
    const int n_qb = (dm.max_seqlen + kBlock - 1) / kBlock;
    const int n = lane & 15, g = lane >> 4;
    const int G = dm.G;
    const float c = dm.scale_log2;

    // the shared list, compacted: entries < 0 or above the own block are dropped (each wavefront keeps its own copy)
    __shared__ int blist[4][64];
    int entry = kNone;
    if (lane < dm.topk) {
        const int x = block_idx[(((int64_t)b * dm.Hkv + h) * n_qb + I) * dm.topk + lane];
        if (x >= 0 && x <= I) entry = x;
    }
    const uint64_t have = __ballot(entry != kNone);
    const int cnt = __popcll(have);
    if (entry != kNone) blist[wave][__popcll(have & ((1ull << lane) - 1ull))] = entry;   // same wavefront reads it back
    bf16x8 qf[kShTok][4];
    f32x4 o[kShTok][8];
    float neg_m[kShTok], l_run[kShTok];
#pragma unroll
    for (int u = 0; u < kShTok; ++u) {
        const int tok = min(t0 + u, L - 1);              // rows past the end compute on a copy and are not written
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            qf[u][ks] = load8(q.ptr + b * q.sb + (int64_t)tok * q.st + (int64_t)(h * G + min(n, G - 1)) * q.sh + 32 * ks + 8 * g);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[u][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        neg_m[u] = __builtin_nanf("");
        l_run[u] = 0.f;
    }
    auto softmax = [&](f32x4 (&s)[2], int u, bf16x8 &pf) __attribute__((always_inline)) {
        float ps = half_probs(s, c, neg_m[u], pf);
        if (__any(!(ps <= kPsumLimit))) {                 // rare: too large, inf, or NaN (no reference yet)
            float tmax = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) tmax = fmaxf(tmax, s[t][j]);
            tmax = xgroup_max(tmax) * c;
            const float old = neg_m[u];
            const float m_new = (old != old) ? tmax : fmaxf(-old, tmax);
            if (m_new > -INFINITY) {
                const float f = (old != old) ? 0.f : fast_exp2(-old - m_new);
                l_run[u] *= f;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[u][dt] *= f;
                neg_m[u] = -m_new;
                ps = half_probs(s, c, -m_new, pf);
            } else {
                ps = 0.f;
                pf = zero8();
            }
        }
        l_run[u] += ps;
    };

    const u32x4 *kv_head = reinterpret_cast<const u32x4 *>(kvp) + ((int64_t)b * dm.Hkv + h) * nb_cap * kPackedBlockU4;
    u32x4 r[8];                                          // this thread's 1/256 of a packed block
    auto fetch = [&](int ci) __attribute__((always_inline)) {
        const int blk = blist[wave][min(ci, cnt - 1)];
        const u32x4 *bp = kv_head + (int64_t)blk * kPackedBlockU4 + tid;
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = bp[256 * i];
    };
    auto stash = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) stage[buf][tid + 256 * i] = r[i];
    };
    if (cnt == 0) return;                                // (cannot happen for a live query block: its own block is forced)
    fetch(0);
    stash(0);
    __syncthreads();
    for (int ci = 0; ci < cnt; ++ci) {
        const int cur = ci & 1;
        fetch(ci + 1);                                   // (a copy of the last block at the end, never used)
        const int blk = blist[wave][ci];
        const int key0 = blk * kBlock;
        const bool edge = blk == I;
        const u32x4 *sb = stage[cur] + lane;
#pragma unroll
        for (int hs = 0; hs < 2; ++hs) {
            // four independent accumulation chains (2 key tiles x 2 tokens) interleaved k-step by k-step: a
            // dependent MFMA then issues three MFMAs after the one it waits for, which covers its latency
            f32x4 s[kShTok][2];
#pragma unroll
            for (int u = 0; u < kShTok; ++u) s[u][0] = s[u][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const u32x4 k0 = sb[(ks * 4 + 2 * hs) * 64], k1 = sb[(ks * 4 + 2 * hs + 1) * 64];
#pragma unroll
                for (int u = 0; u < kShTok; ++u) {
                    s[u][0] = mfma16(__builtin_bit_cast(bf16x8, k0), qf[u][ks], s[u][0]);
                    s[u][1] = mfma16(__builtin_bit_cast(bf16x8, k1), qf[u][ks], s[u][1]);
                }
            }
            bf16x8 pf[kShTok];
#pragma unroll
            for (int u = 0; u < kShTok; ++u) {
                if (edge) {
                    const int tok = t0 + u;
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (key0 + 32 * hs + 16 * t + 4 * g + j > tok) s[u][t][j] = -INFINITY;
                }
                softmax(s[u], u, pf[u]);
            }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                const u32x4 vf = sb[(kFragsPerOperand + dt * 2 + hs) * 64];
#pragma unroll
                for (int u = 0; u < kShTok; ++u) o[u][dt] = mfma16(__builtin_bit_cast(bf16x8, vf), pf[u], o[u][dt]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        stash(cur ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < kShTok; ++u) {
        const int tok = t0 + u;
        if (tok >= L || n >= G) continue;
        const float l_tot = xgroup_sum(l_run[u]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        __bf16 *op = out.ptr + b * out.sb + (int64_t)tok * out.st + (int64_t)(h * G + n) * out.sh + 4 * g;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            bf16x4 rr;
#pragma unroll
            for (int j = 0; j < 4; ++j) rr[j] = (__bf16)(o[u][dt][j] * inv);
            *reinterpret_cast<uint2 *>(op + 16 * dt) = __builtin_bit_cast(uint2, rr);
        }
        if (g == 0)
            lse[((int64_t)b * dm.max_seqlen + tok) * dm.Hq + h * G + n] =
                l_tot > 0.f ? (fast_log2(l_tot) - neg_m[u]) * kLn2 : -INFINITY;
    }
}

size_t attn_prefill_ws_bytes(const Dims &dm) {
    const size_t nb_cap = ((size_t)dm.max_seqlen + kBlock - 1) / kBlock;
    return (size_t)dm.batch * dm.Hkv * nb_cap * kPackedBlockU4 * sizeof(uint4);
}

template <int kTok, int kNU, int kWavesPerSimd>
static void launch_attn_variant(const Dims &dm, Tensor q, const uint4 *kvp, int32_t nb_cap, const int32_t *seqlens,
                                const int32_t *block_idx, Tensor out, float *lse, hipStream_t stream) {
    const int32_t n_tiles = (dm.max_seqlen + 4 * kTok - 1) / (4 * kTok);
    const int64_t n_wg = (int64_t)n_tiles * dm.Hkv * dm.batch;
    hipLaunchKernelGGL((attn_prefill_kernel<kTok, kNU, kWavesPerSimd>), dim3((uint32_t)n_wg), dim3(256), 0, stream,
                       dm, q, kvp, nb_cap, seqlens, block_idx, out, lse, n_tiles);
}

int launch_attn_prefill(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                        const int32_t *block_idx, Tensor out, float *lse, void *ws, hipStream_t stream) {
    const int32_t nb_cap = (dm.max_seqlen + kBlock - 1) / kBlock;
    if (nb_cap <= 0 || dm.batch <= 0) return 0;
    uint4 *kvp = reinterpret_cast<uint4 *>(ws);
    timing_begin("pack_kv_kernel", stream);
    hipLaunchKernelGGL(pack_kv_kernel, dim3(nb_cap, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, k, v,
                       seqlens, kvp, nb_cap);
    timing_end(stream);
    if (dm.shared_q) {                                   // one block list per query block (comparison variant)
        const int32_t n_tiles = (dm.max_seqlen + 7) / 8;
        timing_begin("attn_prefill_shared_kernel", stream);
        hipLaunchKernelGGL(attn_prefill_shared_kernel, dim3((uint32_t)((int64_t)n_tiles * dm.Hkv * dm.batch)), dim3(256),
                           0, stream, dm, q, kvp, nb_cap, seqlens, block_idx, out, lse, n_tiles);
        timing_end(stream);
        return (int)hipGetLastError();
    }
    // 2 tokens per wavefront, ring of 4 units, 2 wavefronts per SIMD: the configuration that keeps
    // the most loads in flight per compute unit within 256 registers per lane
    timing_begin("attn_prefill_kernel", stream);
    launch_attn_variant<2, 4, 2>(dm, q, kvp, nb_cap, seqlens, block_idx, out, lse, stream);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
