/*
 * A client of the C ABI written in plain C99, with no Python and no torch: device memory and
 * copies through the HIP runtime's C interface, the three stages of the path through
 * include/infllmv2.h, every result checked on the host against loops written out here.
 *
 * The case: one sequence of 160 tokens, 16 query heads on 1 key-value head, top-k 8.  160 tokens
 * are 3 blocks, fewer than k, so every token selects all of its blocks and the attention is
 * plain dense causal attention (section 2.1.2: with no more blocks than k the method is vanilla
 * dense attention), which a few loops can check.
 *
 * Test infrastructure: built by tests/c_client/build.py, run by the GPU tests.  Exit status 0 = ok.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "infllmv2.h"

enum { T = 160, HQ = 16, HKV = 1, D = 128, TOPK = 8, M = 64, P = 32, S = 16, NC = (T - P) / S + 1 };

#define CHECK_HIP(x)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));   \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define CHECK_ABI(x)                                                                     \
    do {                                                                                 \
        int32_t s_ = (x);                                                                \
        if (s_ != INFLLMV2_OK) {                                                         \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, infllmv2_status_string(s_)); \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round to nearest, ties to even; every value this program rounds is a small multiple of 2^-9,
 * exact in fp32, so the only rounding is the one to bf16 */
static uint16_t f64_to_bf16(double x) {
    float f = (float)x;
    uint32_t u;
    if ((double)f != x) abort();
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* small exactly representable values from a 32-bit linear congruential generator */
static uint32_t lcg_state = 20250607u;
static uint16_t next_value(void) {
    lcg_state = lcg_state * 1664525u + 1013904223u;
    int v = (int)((lcg_state >> 16) % 33u) - 16; /* -16 .. 16 */
    return f64_to_bf16((double)v / 16.0);
}

int main(void) {
    static uint16_t q[T][HQ][D], k[T][D], v[T][D], ck[NC][D], out[T][HQ][D];
    static float lse[T][HQ];
    static int32_t idx[T][TOPK];
    int n_dev = 0;
    CHECK_HIP(hipGetDeviceCount(&n_dev));
    if (n_dev < 1) {
        fprintf(stderr, "no GPU\n");
        return 2;
    }
    for (int t = 0; t < T; ++t) {
        for (int c = 0; c < D; ++c) {
            k[t][c] = next_value();
            v[t][c] = next_value();
        }
        for (int h = 0; h < HQ; ++h)
            for (int c = 0; c < D; ++c) q[t][h][c] = next_value();
    }
    infllmv2_params prm;
    memset(&prm, 0, sizeof prm);
    prm.head_dim = D;
    prm.n_q_heads = HQ;
    prm.n_kv_heads = HKV;
    prm.block_size = M;
    prm.kernel_size = P;
    prm.kernel_stride = S;
    prm.topk = TOPK;
    prm.n_init_blocks = 1;
    prm.n_local_blocks = 2;
    prm.softmax_scale = 1.0f / sqrtf((float)D);
    prm.lse_coarse_ratio = 1;

    void *dq, *dk, *dv, *dck, *dout, *dlse, *didx, *dsl, *dws = NULL;
    const int32_t seqlen = T;
    CHECK_HIP(hipMalloc(&dq, sizeof q));
    CHECK_HIP(hipMalloc(&dk, sizeof k));
    CHECK_HIP(hipMalloc(&dv, sizeof v));
    CHECK_HIP(hipMalloc(&dck, sizeof ck));
    CHECK_HIP(hipMalloc(&dout, sizeof out));
    CHECK_HIP(hipMalloc(&dlse, sizeof lse));
    CHECK_HIP(hipMalloc(&didx, sizeof idx));
    CHECK_HIP(hipMalloc(&dsl, sizeof seqlen));
    CHECK_HIP(hipMemcpy(dq, q, sizeof q, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dk, k, sizeof k, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dv, v, sizeof v, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dsl, &seqlen, sizeof seqlen, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(dck, 0, sizeof ck));
    size_t ws_sel = infllmv2_workspace_bytes(INFLLMV2_OP_SELECT_PREFILL, &prm, 1, T);
    size_t ws_att = infllmv2_workspace_bytes(INFLLMV2_OP_ATTN_PREFILL, &prm, 1, T);
    size_t ws_bytes = ws_sel > ws_att ? ws_sel : ws_att;
    if (ws_bytes > 0) CHECK_HIP(hipMalloc(&dws, ws_bytes));

    const infllmv2_tensor tq = {dq, (int64_t)T * HQ * D, D, (int64_t)HQ * D};    /* [b, t, hq, c] */
    const infllmv2_tensor to = {dout, (int64_t)T * HQ * D, D, (int64_t)HQ * D};
    const infllmv2_tensor tk = {dk, (int64_t)T * D, (int64_t)T * D, D};          /* [b, h, t, c] */
    const infllmv2_tensor tv = {dv, (int64_t)T * D, (int64_t)T * D, D};
    const infllmv2_tensor tck = {dck, (int64_t)NC * D, (int64_t)NC * D, D};

    CHECK_ABI(infllmv2_compress_keys(&prm, &tk, (const int32_t *)dsl, 1, T, 0, &tck, NULL));
    CHECK_ABI(infllmv2_select_blocks(&prm, INFLLMV2_MODE_PREFILL, &tq, &tck, (const int32_t *)dsl, 1, T,
                                     (int32_t *)didx, dws, ws_bytes, NULL));
    CHECK_ABI(infllmv2_sparse_attn_prefill(&prm, &tq, &tk, &tv, (const int32_t *)dsl, 1, T, (const int32_t *)didx,
                                           &to, (float *)dlse, dws, ws_bytes, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(ck, dck, sizeof ck, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(idx, didx, sizeof idx, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(out, dout, sizeof out, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(lse, dlse, sizeof lse, hipMemcpyDeviceToHost));

    int bad = 0;
    /* stage 1: mean of 32 rows, one rounding (section 2.1.2 "Semantic Kernels") */
    for (int j = 0; j < NC; ++j)
        for (int c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int t = j * S; t < j * S + P; ++t) acc += (double)bf16_to_f32(k[t][c]);
            if (ck[j][c] != f64_to_bf16(acc / P)) ++bad;
        }
    if (bad) {
        fprintf(stderr, "compressed keys: %d elements differ\n", bad);
        return 1;
    }
    /* stage 2: fewer blocks than k, so every block up to the token's own, ascending, then -1 */
    for (int t = 0; t < T; ++t) {
        const int n_blk = t / M + 1;
        for (int e = 0; e < TOPK; ++e)
            if (idx[t][e] != (e < n_blk ? e : -1)) ++bad;
    }
    if (bad) {
        fprintf(stderr, "block lists: %d entries differ\n", bad);
        return 1;
    }
    /* stage 3: dense causal attention */
    double worst_o = 0.0, worst_l = 0.0;
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < HQ; ++h) {
            double z[T], m = -INFINITY, den = 0.0, o[D];
            for (int u = 0; u <= t; ++u) {
                double a = 0.0;
                for (int c = 0; c < D; ++c) a += (double)bf16_to_f32(q[t][h][c]) * (double)bf16_to_f32(k[u][c]);
                z[u] = a * (double)prm.softmax_scale;
                if (z[u] > m) m = z[u];
            }
            memset(o, 0, sizeof o);
            for (int u = 0; u <= t; ++u) {
                const double p = exp(z[u] - m);
                den += p;
                for (int c = 0; c < D; ++c) o[c] += p * (double)bf16_to_f32(v[u][c]);
            }
            for (int c = 0; c < D; ++c) {
                const double e = fabs((double)bf16_to_f32(out[t][h][c]) - o[c] / den);
                if (e > worst_o) worst_o = e;
            }
            const double el = fabs((double)lse[t][h] - (m + log(den)));
            if (el > worst_l) worst_l = el;
        }
    printf("abi_client: compressed keys and block lists exact; attention max|dO| %.3e max|dLSE| %.3e\n", worst_o,
           worst_l);
    if (!(worst_o <= 2e-2) || !(worst_l <= 1e-5)) return 1;

    /* decode: the last token once more, as the one query of a decode step over the same cache -- stage 2 in
     * decode mode, then infllmv2_sparse_attn_decode; the same row as the prefill above, from other kernels */
    {
        static uint16_t out_d[HQ][D];
        static float lse_d[HQ];
        static int32_t idx_d[TOPK];
        void *dout_d, *dlse_d, *didx_d, *dws_d = NULL;
        size_t ws_ds = infllmv2_workspace_bytes(INFLLMV2_OP_SELECT_DECODE, &prm, 1, T);
        size_t ws_da = infllmv2_workspace_bytes(INFLLMV2_OP_ATTN_DECODE, &prm, 1, T);
        size_t ws_d = ws_ds > ws_da ? ws_ds : ws_da;
        CHECK_HIP(hipMalloc(&dout_d, sizeof out_d));
        CHECK_HIP(hipMalloc(&dlse_d, sizeof lse_d));
        CHECK_HIP(hipMalloc(&didx_d, sizeof idx_d));
        if (ws_d > 0) CHECK_HIP(hipMalloc(&dws_d, ws_d));
        const infllmv2_tensor tq_d = {(uint16_t *)dq + (size_t)(T - 1) * HQ * D, (int64_t)HQ * D, D, (int64_t)HQ * D};
        const infllmv2_tensor to_d = {dout_d, (int64_t)HQ * D, D, (int64_t)HQ * D};
        CHECK_ABI(infllmv2_select_blocks(&prm, INFLLMV2_MODE_DECODE, &tq_d, &tck, (const int32_t *)dsl, 1, T,
                                         (int32_t *)didx_d, dws_d, ws_d, NULL));
        CHECK_ABI(infllmv2_sparse_attn_decode(&prm, &tq_d, &tk, &tv, (const int32_t *)dsl, 1, T,
                                              (const int32_t *)didx_d, &to_d, (float *)dlse_d, dws_d, ws_d, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(idx_d, didx_d, sizeof idx_d, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(out_d, dout_d, sizeof out_d, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(lse_d, dlse_d, sizeof lse_d, hipMemcpyDeviceToHost));
        for (int e = 0; e < TOPK; ++e)
            if (idx_d[e] != idx[T - 1][e]) ++bad;
        if (bad) {
            fprintf(stderr, "decode block list differs from the prefill row\n");
            return 1;
        }
        double wo = 0.0, wl = 0.0;
        for (int h = 0; h < HQ; ++h) {
            for (int c = 0; c < D; ++c) {
                const double e = fabs((double)bf16_to_f32(out_d[h][c]) - (double)bf16_to_f32(out[T - 1][h][c]));
                if (e > wo) wo = e;
            }
            const double el = fabs((double)lse_d[h] - (double)lse[T - 1][h]);
            if (el > wl) wl = el;
        }
        printf("abi_client: decode of the last token vs its prefill row max|dO| %.3e max|dLSE| %.3e\n", wo, wl);
        /* both sides are within 2e-2 / 1e-5 of the exact row (checked above for the prefill side) */
        if (!(wo <= 2e-2) || !(wl <= 2e-5)) return 1;
        (void)hipFree(dout_d); (void)hipFree(dlse_d); (void)hipFree(didx_d);
        if (dws_d) (void)hipFree(dws_d);
    }
    (void)hipFree(dq); (void)hipFree(dk); (void)hipFree(dv); (void)hipFree(dck); (void)hipFree(dout);
    (void)hipFree(dlse); (void)hipFree(didx); (void)hipFree(dsl);
    if (dws) (void)hipFree(dws);
    printf("abi_client ok\n");
    return 0;
}
