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
// kPrefetch: keep the next operand's 16 fragments in flight while computing on the current one
// (K during the value phase, V during the score phase); costs 64 more registers per lane.
template <int kTok, bool kPrefetch, int kWavesPerSimd>
__global__ __launch_bounds__(256, kWavesPerSimd) void attn_prefill_kernel(Dims dm, Tensor q, const uint4 *__restrict__ kvp,
                                                            int32_t nb_cap,
                                                            const int32_t *__restrict__ seqlens,
                                                            const int32_t *__restrict__ block_idx,
                                                            Tensor out, float *__restrict__ lse,
                                                            int32_t n_tiles) {
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

    bf16x8 qf[kTok][4];
    f32x4 o[kTok][8];
    float m_run[kTok], l_run[kTok];
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
        m_run[u] = -INFINITY;
        l_run[u] = 0.f;
        int e = 0x7fffffff;
        if (live && lane < dm.topk) {
            int x = block_idx[(((int64_t)b * dm.Hkv + h) * dm.max_seqlen + tok) * dm.topk + lane];
            if (x >= 0 && x <= b_own) e = x;
        }
        own[u] = e;
    }
    const uint4 *kv_head = kvp + ((int64_t)b * dm.Hkv + h) * nb_cap * kPackedBlockU4;   // uniform

    auto next_block = [&](int cur) {
        int cand = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < kTok; ++u) {
            int e = own[u] > cur ? own[u] : 0x7fffffff;
            cand = e < cand ? e : cand;
        }
        return __builtin_amdgcn_readfirstlane(wave_min_i32(cand));   // wave-uniform: scalar addressing
    };

    int blk = next_block(-1);
    uint4 kf[16];
    if (kPrefetch && blk != 0x7fffffff) {
        const uint4 *p = kv_head + (int64_t)blk * kPackedBlockU4;
#pragma unroll
        for (int f = 0; f < 16; ++f) kf[f] = p[f * 64 + lane];
    }
    while (blk != 0x7fffffff) {
        uint4 vf[16];
        if (kPrefetch) {           // value fragments of this block: in flight during the score phase
            const uint4 *p = kv_head + (int64_t)blk * kPackedBlockU4 + kFragsPerOperand * 64;
#pragma unroll
            for (int f = 0; f < 16; ++f) vf[f] = p[f * 64 + lane];
        } else {
            const uint4 *p = kv_head + (int64_t)blk * kPackedBlockU4;
#pragma unroll
            for (int f = 0; f < 16; ++f) kf[f] = p[f * 64 + lane];
        }
        bool member[kTok];
#pragma unroll
        for (int u = 0; u < kTok; ++u) member[u] = __ballot(own[u] == blk) != 0ull;
        const int nxt = next_block(blk);
        const int key0 = blk * kBlock;
        const bool edge = (blk == b_own) || (key0 + kBlock > L);

        // ---- S^T = K . Q^T, online softmax, P^T packed to bf16 in MFMA B layout -----------------
        bf16x8 pf[kTok][2];
#pragma unroll
        for (int u = 0; u < kTok; ++u) {
            if (!member[u]) continue;
            f32x4 s[4];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) s[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    s[mt] = mfma16(__builtin_bit_cast(bf16x8, kf[ks * 4 + mt]), qf[u][ks], s[mt]);
            const int tok = t0 + u;
            float mx = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float x = s[mt][j] * dm.scale_log2;
                    if (edge && key0 + 16 * mt + 4 * g + j > tok) x = -INFINITY;
                    s[mt][j] = x;
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
                    float p = fast_exp2(s[mt][j] - m_use);
                    s[mt][j] = p;
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
                    p8[j] = (__bf16)s[2 * kk][j];
                    p8[4 + j] = (__bf16)s[2 * kk + 1][j];
                }
                pf[u][kk] = p8;
            }
        }
        if (kPrefetch) {           // key fragments of the next block: in flight during the value phase
            if (nxt != 0x7fffffff) {
                const uint4 *p = kv_head + (int64_t)nxt * kPackedBlockU4;
#pragma unroll
                for (int f = 0; f < 16; ++f) kf[f] = p[f * 64 + lane];
            }
        } else {
            const uint4 *p = kv_head + (int64_t)blk * kPackedBlockU4 + kFragsPerOperand * 64;
#pragma unroll
            for (int f = 0; f < 16; ++f) vf[f] = p[f * 64 + lane];
        }
        // ---- O^T += V^T . P^T ----------------------------------------------------------------------
#pragma unroll
        for (int u = 0; u < kTok; ++u) {
            if (!member[u]) continue;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
                    o[u][dt] = mfma16(__builtin_bit_cast(bf16x8, vf[dt * 2 + kk]), pf[u][kk], o[u][dt]);
        }
        blk = nxt;
    }

    // ---- normalise and write: lane holds channels 16*dt + 4*g .. +3 of head n ------------------
#pragma unroll
    for (int u = 0; u < kTok; ++u) {
        const int tok = t0 + u;
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

size_t attn_prefill_ws_bytes(const Dims &dm) {
    const size_t nb_cap = ((size_t)dm.max_seqlen + kBlock - 1) / kBlock;
    return (size_t)dm.batch * dm.Hkv * nb_cap * kPackedBlockU4 * sizeof(uint4);
}

int launch_attn_prefill(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                        const int32_t *block_idx, Tensor out, float *lse, void *ws, hipStream_t stream) {
    constexpr int kTok = 2;
    const int32_t nb_cap = (dm.max_seqlen + kBlock - 1) / kBlock;
    if (nb_cap <= 0 || dm.batch <= 0) return 0;
    uint4 *kvp = reinterpret_cast<uint4 *>(ws);
    timing_begin("pack_kv_kernel", stream);
    hipLaunchKernelGGL(pack_kv_kernel, dim3(nb_cap, dm.Hkv, dm.batch), dim3(256), 0, stream, dm, k, v,
                       seqlens, kvp, nb_cap);
    timing_end(stream);
    const int32_t n_tiles = (dm.max_seqlen + 4 * kTok - 1) / (4 * kTok);
    const int64_t n_wg = (int64_t)n_tiles * dm.Hkv * dm.batch;
    timing_begin("attn_prefill_kernel", stream);
    hipLaunchKernelGGL((attn_prefill_kernel<kTok, false, 2>), dim3((uint32_t)n_wg), dim3(256), 0, stream, dm, q, kvp,
                       nb_cap, seqlens, block_idx, out, lse, n_tiles);
    timing_end(stream);
    return (int)hipGetLastError();
}

}  // namespace infllmv2
