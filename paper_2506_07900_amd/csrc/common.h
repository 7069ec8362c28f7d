// Device-side helpers shared by the HIP kernels (gfx950 / CDNA4 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/infllmv2.h"

namespace infllmv2 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Geometry the kernels are specialised for ("Hyper-Parameter Recommendation": p=32, s=16; m=64).
constexpr int kHeadDim = 128;
constexpr int kBlock = 64;    // m
constexpr int kKernel = 32;   // p
constexpr int kStride = 16;   // s
constexpr int kMaxTopk = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kScoreFloor = 7.888609052210118e-31f;  // 2^-100, floor of a relevance score
constexpr float kScoreCeil = 1.2676506002282294e30f;   // 2^100, ceiling (only the approximate LSE can reach it)

// Host+device view of the call: everything a kernel needs besides its own buffers.
struct Dims {
    int32_t Hq, Hkv, G;
    int32_t topk, n_init, n_local;
    int32_t batch, max_seqlen;
    float scale_log2;   // softmax_scale * log2(e)
    int32_t rho;        // coarse / fine kernel stride of the approximate log-sum-exp; 1 = exact
    int32_t n_q;        // decode-side kernels: query tokens per sequence (1 = plain decode, n = draft verification)
    int32_t shared_q;   // prefill selection: 1 = one block set per 64-token query block (comparison variant)
};

struct Tensor {          // strides in elements
    __bf16 *ptr;
    int64_t sb, sh, st;
};

struct AppendArgs {      // the cache append folded into the first kernel of a fused decode step
    Tensor k_new, v_new, k, v;
};
struct AttendArgs {      // the per-block attention folded into the top-k kernel of a fused decode step
    Tensor k, v;
    const uint64_t *tree_mask;                        // verification only, else null
    bool fused;                                       // out: false = only the top-k ran (too many rows to repeat it per block)
    float *o_part;
    float2 *ml_part;
};

// Number of complete semantic kernels of a sequence of l tokens (p=32, s=16).
__host__ __device__ inline int32_t num_kernels(int32_t l) {
    return l < kKernel ? 0 : (l - kKernel) / kStride + 1;
}

// Number of coarse kernels (ratio rho) all of whose fine kernels rho*c + 2r, r < rho, lie among the
// first n fine kernels ("Efficient Top-K Implementation": coarse-grained semantic kernels).
__host__ __device__ inline int32_t num_coarse(int32_t n, int32_t rho) {
    return n < 2 * rho - 1 ? 0 : (n - (2 * rho - 1)) / rho + 1;
}

// fp64 -> bf16, round to nearest even with a single rounding: first round-to-odd to fp32
// (24 bits keep a sticky bit), then nearest-even to 8 bits.
__device__ inline uint16_t f64_to_bf16_rne(double x) {
    float f = (float)x;
    uint32_t u = __float_as_uint(f);
    double fd = (double)f;
    if (fd != x) {
        if (fabs(fd) > fabs(x)) u -= 1u;   // back to the truncated magnitude
        u |= 1u;                           // inexact: make the last bit odd
    }
    uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(r >> 16);
}

// 16x16x32 bf16 MFMA, D = A*B + C.
//   A is 16(M) x 32(K): lane l holds row l%16, k = 8*(l/16) .. 8*(l/16)+7
//   B is 32(K) x 16(N): lane l holds column l%16, same k range
//   C/D is 16 x 16:     lane l holds column l%16, rows 4*(l/16) .. 4*(l/16)+3
__device__ inline f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ inline bf16x8 load8(const __bf16 *p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(p));
}

__device__ inline bf16x8 zero8() {
    uint4 z = {0u, 0u, 0u, 0u};
    return __builtin_bit_cast(bf16x8, z);
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Reduce over the four 16-lane groups of a wavefront (lanes l, l^16, l^32, l^48).
__device__ inline float xgroup_max(float v) {
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}
__device__ inline float xgroup_sum(float v) {
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// Top-k by counting (used by the pick kernels).  An element is the 64-bit word
// key << 32 | ~block: larger word = better element, ties go to the lower block index.
constexpr uint64_t kPickValid = 1ull << 32;               // smallest word of a real candidate

// number of words in w[0..n) (n a multiple of 4, 16-byte aligned) that are larger than x; sixteen
// words per step, all loaded before any is compared (a step costs one LDS latency, not eight)
__device__ inline int count_larger(const uint64_t *w, int n, uint64_t x) {
    int c0 = 0, c1 = 0;
    int j = 0;
    for (; j + 16 <= n; j += 16) {
        ulonglong2 a[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = *reinterpret_cast<const ulonglong2 *>(w + j + 2 * i);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            c0 += a[i].x > x ? 1 : 0;
            c1 += a[i].y > x ? 1 : 0;
        }
    }
    for (; j < n; j += 4) {
        const ulonglong2 a = *reinterpret_cast<const ulonglong2 *>(w + j);
        const ulonglong2 bq = *reinterpret_cast<const ulonglong2 *>(w + j + 2);
        c0 += (a.x > x ? 1 : 0) + (bq.x > x ? 1 : 0);
        c1 += (a.y > x ? 1 : 0) + (bq.y > x ? 1 : 0);
    }
    return c0 + c1;
}

// The word of block j with the given score: candidates are the blocks n_init .. jc_max; a candidate
// without any visible kernel (-inf) gets key 1, below every real score (>= 2^-100) and above "none".
__device__ inline uint64_t pick_element(float score, int j, int n_init, int jc_max) {
    const uint32_t kj = score == -INFINITY ? 1u : __float_as_uint(score);
    const uint32_t key = (j >= n_init && j <= jc_max) ? kj : 0u;
    return ((uint64_t)key << 32) | (uint32_t)~j;
}

// Wavefront top-n of distinct 64-bit words, no serial rounds.  Lane l brings NE words; words below
// kPickValid are not candidates.  Returns in lane c < n the c-th largest candidate (0 when there are
// fewer than c + 1); n <= 64.  An element of the top n can only sit in a lane whose own maximum is
// among the n largest lane maxima, and it is at least tau, the n-th largest lane maximum: rank the 64
// lane maxima by counting, let the n best lanes publish their words >= tau (a handful), rank those by
// counting.  lds: 64 + topk_cand_cap(n, NE) words that belong to this wavefront alone.
__host__ __device__ inline int topk_cand_cap(int n, int ne) { return (n * ne + 3) & ~3; }

template <int NE>
__device__ inline uint64_t wave_topk(const uint64_t (&el)[NE], int n, uint64_t *lds, int lane) {
    uint64_t *tmax = lds, *cand = lds + 64;
    uint64_t best = 0ull;
#pragma unroll
    for (int s = 0; s < NE; ++s) best = el[s] > best ? el[s] : best;
    tmax[lane] = best;
    __builtin_amdgcn_wave_barrier();
    const bool real = best >= kPickValid;
    const int lrank = count_larger(tmax, 64, best);
    const bool finalist = real && lrank < n;
    uint64_t tau = kPickValid;                            // when fewer than n lanes hold a candidate
    const uint64_t who = __ballot(real && lrank == n - 1);
    if (who) {
        const int src = __builtin_ctzll(who);
        tau = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(best >> 32), src) << 32) |
              (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)best, src);
    }
    int n_cand = 0;
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int s = 0; s < NE; ++s) {
        const bool pub = finalist && el[s] >= tau;
        const uint64_t m = __ballot(pub);
        if (pub) cand[n_cand + __popcll(m & below)] = el[s];
        n_cand += __popcll(m);
    }
    const int n_cand4 = (n_cand + 3) & ~3;                // <= topk_cand_cap(n, NE)
    if (lane < n_cand4 - n_cand) cand[n_cand + lane] = 0ull;
    tmax[lane] = 0ull;                                    // the ranks are known: reuse as the result row
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < n_cand; i += 64) {
        const uint64_t e = cand[i];
        const int beaten = count_larger(cand, n_cand4, e);
        if (beaten < n) tmax[beaten] = e;
    }
    __builtin_amdgcn_wave_barrier();
    const uint64_t res = lane < n ? tmax[lane] : 0ull;
    __builtin_amdgcn_wave_barrier();
    return res;
}

// The row of selected blocks of one query: lane c < n_pick brings a picked candidate block, the forced
// blocks (the first n_init and lo_local .. b_own) are added, and the n_sel blocks are written in
// ascending order, padded with -1 up to topk.
__device__ inline void write_block_row(int picked, int n_pick, int n_sel, int n_init, int lo_local, int topk,
                                       int32_t *__restrict__ o, int lane) {
    int mine = 0x7fffffff;
    if (lane < n_pick) mine = picked;
    else if (lane < n_sel) {
        const int f = lane - n_pick;
        mine = f < n_init ? f : lo_local + (f - n_init);
    }
    int rank = 0;                                         // number of selected blocks below mine
    for (int e = 0; e < n_sel; ++e) rank += __builtin_amdgcn_readlane(mine, e) < mine ? 1 : 0;
    if (lane < n_sel) o[rank] = mine;
    else if (lane < topk) o[lane] = -1;
}

// Per-kernel timing of the bench-only build (INFLLMV2_TIMING, see timing.hip): every launch is bracketed
// by HIP events on its stream while infllmv2_timing_enable is on.  The production build compiles the
// hooks away.
#ifdef INFLLMV2_TIMING
void timing_begin(const char *kernel_name, hipStream_t stream);
void timing_end(hipStream_t stream);
#else
inline void timing_begin(const char *, hipStream_t) {}
inline void timing_end(hipStream_t) {}
#endif

// Launchers implemented in the .hip files; each returns a hipError_t as int.
int launch_compress_keys(const Dims &dm, Tensor k, Tensor ck, const int32_t *seqlens,
                         int32_t n_new_tokens, hipStream_t stream);
int launch_append_kv(const Dims &dm, Tensor k_new, Tensor v_new, Tensor k, Tensor v, const Tensor *ck,
                     const int32_t *seqlens, hipStream_t stream);   // dm.n_q rows per sequence
int launch_select_prefill(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                          int32_t *block_idx, void *ws, hipStream_t stream, float *scores_out = nullptr,
                          int32_t scores_pitch = 0);
size_t select_prefill_ws_bytes(const Dims &dm);
int launch_select_prefill16(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                            int32_t *block_idx, void *ws, hipStream_t stream, float *scores_out = nullptr,
                            int32_t scores_pitch = 0);
size_t select_prefill16_ws_bytes(const Dims &dm);
int32_t select_scores_pitch(const Dims &dm);
size_t select_scores_bytes(const Dims &dm);
size_t select_shared_scores_bytes(const Dims &dm);
int launch_select_pick(const Dims &dm, const int32_t *seqlens, const float *R, int32_t nb_cap,
                       int32_t *block_idx, hipStream_t stream);
int launch_select_decode(const Dims &dm, Tensor q, Tensor ck, const int32_t *seqlens,
                         int32_t *block_idx, void *ws, hipStream_t stream, const AppendArgs *append = nullptr,
                         AttendArgs *attend = nullptr);
int launch_decode_step(const Dims &dm, Tensor q, Tensor ck, const AppendArgs &append, const int32_t *seqlens,
                       int32_t *block_idx, Tensor out, float *lse, void *ws_select, void *ws_attn,
                       hipStream_t stream);
int launch_verify_step(const Dims &dm, Tensor q, Tensor ck, const AppendArgs &append, const int32_t *seqlens,
                       const uint64_t *tree_mask, int32_t *block_idx, Tensor out, float *lse, void *ws_select,
                       void *ws_attn, hipStream_t stream);
size_t select_decode_ws_bytes(const Dims &dm);
int launch_attn_prefill(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                        const int32_t *block_idx, Tensor out, float *lse, void *ws, hipStream_t stream);
size_t attn_prefill_ws_bytes(const Dims &dm);
int launch_attn_decode(const Dims &dm, Tensor q, Tensor k, Tensor v, const int32_t *seqlens,
                       const int32_t *block_idx, const uint64_t *tree_mask, Tensor out, float *lse, void *ws,
                       hipStream_t stream);
size_t attn_decode_ws_bytes(const Dims &dm);
int launch_attn_bwd(const Dims &dm, Tensor q, Tensor k, Tensor v, Tensor out, Tensor dout, const float *lse,
                    const int32_t *seqlens, const int32_t *block_idx, Tensor dq, Tensor dk, Tensor dv, void *ws,
                    hipStream_t stream);
size_t attn_bwd_ws_bytes(const Dims &dm);
int32_t validate_attn_decode(const infllmv2_params *prm, const infllmv2_tensor *q, const infllmv2_tensor *k,
                             const infllmv2_tensor *v, const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                             const int32_t *block_idx, const infllmv2_tensor *out, const float *lse, Dims *dm,
                             Tensor *tq, Tensor *tk, Tensor *tv, Tensor *tout);
int launch_probes(void *buf, size_t buf_bytes, double *mfma_flops, double *stream_bytes, hipStream_t stream);
int launch_probes_detail(void *buf, size_t buf_bytes, double *work, hipStream_t stream);

}  // namespace infllmv2
