/* Runs every entry point of the C oracle on small seeded inputs with every buffer on the heap at its exact
 * size, so that AddressSanitizer and UndefinedBehaviorSanitizer (this file and oracle/infllmv2_oracle.c are
 * compiled together with -fsanitize=address,undefined) see any out-of-bounds access, overflow or misuse.
 * Lengths cover the edges: shorter than one semantic kernel, exactly one, a ragged tail, several blocks.
 * Checks no values (tests/test_oracle_pins.py does); exit status 0 and "oracle_san ok" = clean run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int32_t oracle_num_kernels(int32_t l, int32_t p, int32_t s);
int32_t oracle_num_coarse(int32_t n, int32_t rho);
int32_t oracle_compress_keys(const uint16_t *k_bits, int32_t Hkv, int32_t l, int32_t d, int32_t p, int32_t s,
                             double *ck_f64, uint16_t *ck_bits);
int32_t oracle_coarse_kernels(const uint16_t *ck_bits, int32_t Hkv, int32_t n_c, int32_t d, int32_t rho,
                              double *ckc_f64, uint16_t *ckc_bits);
void oracle_kernel_scores(const uint16_t *q_bits, const uint16_t *ck_bits, const int32_t *pos, int32_t Tq,
                          int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c, int32_t p, int32_t s, double scale,
                          double *r_out);
void oracle_kernel_scores_coarse(const uint16_t *q_bits, const uint16_t *ck_bits, const uint16_t *ckc_bits,
                                 const int32_t *pos, int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c,
                                 int32_t n_cc, int32_t p, int32_t s, int32_t rho, double scale, double *r_out,
                                 double *lse_out);
void oracle_select_blocks(const uint16_t *q_bits, const uint16_t *ck_bits, const int32_t *pos, int32_t Tq,
                          int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c, int32_t m, int32_t p, int32_t s,
                          int32_t topk, int32_t n_init, int32_t n_local, double scale, int32_t *block_idx,
                          double *margins, double *R_out, int32_t nb_cap);
void oracle_select_blocks_coarse(const uint16_t *q_bits, const uint16_t *ck_bits, const uint16_t *ckc_bits,
                                 const int32_t *pos, int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c,
                                 int32_t n_cc, int32_t m, int32_t p, int32_t s, int32_t topk, int32_t n_init,
                                 int32_t n_local, int32_t rho, double scale, int32_t *block_idx, double *margins,
                                 double *R_out, int32_t nb_cap);
void oracle_sparse_attn(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits, const int32_t *pos,
                        const int32_t *block_idx, int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t l,
                        int32_t m, int32_t topk, double scale, double *out, double *lse, double *probs_sum);
void oracle_sparse_attn_tree(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits,
                             const int32_t *block_idx, const uint64_t *tree_mask, int32_t n, int32_t l_ctx,
                             int32_t Hq, int32_t Hkv, int32_t d, int32_t l, int32_t m, int32_t topk, double scale,
                             double *out, double *lse);
void oracle_sparse_attn_bwd(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits,
                            const uint16_t *dout_bits, const int32_t *pos, const int32_t *block_idx, int32_t Tq,
                            int32_t Hq, int32_t Hkv, int32_t d, int32_t l, int32_t m, int32_t topk, double scale,
                            double *dq, double *dk, double *dv, double *dq_mag, double *dk_mag, double *dv_mag);
uint16_t oracle_f64_to_bf16(double x);
double oracle_bf16_to_f64(uint16_t b);

static uint32_t rng = 2506u;
static double unit(void) {                        /* uniform in (-1, 1) */
    rng = rng * 1664525u + 1013904223u;
    return ((double)(rng >> 8) / 8388608.0) - 1.0;
}
static void *xalloc(size_t n, size_t sz) {        /* exact size, at least one element so that it is never NULL */
    void *p = calloc(n ? n : 1, sz);
    if (!p) exit(3);
    return p;
}
static uint16_t *random_bits(size_t n) {
    uint16_t *a = (uint16_t *)xalloc(n, sizeof *a);
    for (size_t i = 0; i < n; ++i) a[i] = oracle_f64_to_bf16(unit() * 2.0);
    return a;
}

static void run_case(int32_t l, int32_t Hq, int32_t Hkv, int32_t topk, int32_t n_init, int32_t n_local, int32_t rho) {
    const int32_t d = 16, m = 64, p = 32, s = 16, G = Hq / Hkv;
    const double scale = 1.0 / sqrt((double)d);
    const int32_t n_c = oracle_num_kernels(l, p, s), n_cc = oracle_num_coarse(n_c, rho);
    const int32_t nb = (l + m - 1) / m;
    uint16_t *q = random_bits((size_t)l * Hq * d), *k = random_bits((size_t)Hkv * l * d), *v = random_bits((size_t)Hkv * l * d);
    uint16_t *dout = random_bits((size_t)l * Hq * d);
    double *ck64 = (double *)xalloc((size_t)Hkv * n_c * d, sizeof(double));
    uint16_t *ckb = (uint16_t *)xalloc((size_t)Hkv * n_c * d, sizeof(uint16_t));
    if (oracle_compress_keys(k, Hkv, l, d, p, s, ck64, ckb) != n_c) exit(4);
    double *cc64 = (double *)xalloc((size_t)Hkv * n_cc * d, sizeof(double));
    uint16_t *ccb = (uint16_t *)xalloc((size_t)Hkv * n_cc * d, sizeof(uint16_t));
    if (oracle_coarse_kernels(ckb, Hkv, n_c, d, rho, cc64, ccb) != n_cc) exit(4);
    int32_t *pos = (int32_t *)xalloc((size_t)l, sizeof(int32_t));
    for (int32_t t = 0; t < l; ++t) pos[t] = t;
    double *r = (double *)xalloc((size_t)Hkv * l * n_c, sizeof(double));
    double *lse_c = (double *)xalloc((size_t)Hkv * l * G, sizeof(double));
    oracle_kernel_scores(q, ckb, pos, l, Hq, Hkv, d, n_c, p, s, scale, r);
    oracle_kernel_scores_coarse(q, ckb, ccb, pos, l, Hq, Hkv, d, n_c, n_cc, p, s, rho, scale, r, lse_c);
    int32_t *idx = (int32_t *)xalloc((size_t)Hkv * l * topk, sizeof(int32_t));
    double *margins = (double *)xalloc((size_t)Hkv * l * 2, sizeof(double));
    double *R = (double *)xalloc((size_t)Hkv * l * nb, sizeof(double));
    oracle_select_blocks_coarse(q, ckb, ccb, pos, l, Hq, Hkv, d, n_c, n_cc, m, p, s, topk, n_init, n_local, rho, scale,
                                idx, margins, R, nb);
    oracle_select_blocks(q, ckb, pos, l, Hq, Hkv, d, n_c, m, p, s, topk, n_init, n_local, scale, idx, NULL, NULL, nb);
    oracle_select_blocks(q, ckb, pos, l, Hq, Hkv, d, n_c, m, p, s, topk, n_init, n_local, scale, idx, margins, R, nb);
    double *out = (double *)xalloc((size_t)l * Hq * d, sizeof(double));
    double *lse = (double *)xalloc((size_t)l * Hq, sizeof(double));
    double *ps = (double *)xalloc((size_t)l * Hq, sizeof(double));
    oracle_sparse_attn(q, k, v, pos, idx, l, Hq, Hkv, d, l, m, topk, scale, out, lse, ps);
    oracle_sparse_attn(q, k, v, pos, idx, l, Hq, Hkv, d, l, m, topk, scale, out, lse, NULL);
    double *dq = (double *)xalloc((size_t)l * Hq * d, sizeof(double)), *dqm = (double *)xalloc((size_t)l * Hq * d, sizeof(double));
    double *dk = (double *)xalloc((size_t)Hkv * l * d, sizeof(double)), *dkm = (double *)xalloc((size_t)Hkv * l * d, sizeof(double));
    double *dv = (double *)xalloc((size_t)Hkv * l * d, sizeof(double)), *dvm = (double *)xalloc((size_t)Hkv * l * d, sizeof(double));
    oracle_sparse_attn_bwd(q, k, v, dout, pos, idx, l, Hq, Hkv, d, l, m, topk, scale, dq, dk, dv, dqm, dkm, dvm);
    oracle_sparse_attn_bwd(q, k, v, dout, pos, idx, l, Hq, Hkv, d, l, m, topk, scale, dq, dk, dv, NULL, NULL, NULL);
    /* draft verification: the last n tokens are the drafted ones, a chain mask */
    const int32_t n = l < 5 ? l : 5, l_ctx = l - n;
    uint64_t *mask = (uint64_t *)xalloc((size_t)n, sizeof(uint64_t));
    int32_t *idx_t = (int32_t *)xalloc((size_t)Hkv * n * topk, sizeof(int32_t));
    for (int32_t t = 0; t < n; ++t) mask[t] = (2ull << t) - 1ull;
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t t = 0; t < n; ++t)
            memcpy(idx_t + ((size_t)h * n + t) * topk, idx + ((size_t)h * l + l_ctx + t) * topk, sizeof(int32_t) * (size_t)topk);
    double *out_t = (double *)xalloc((size_t)n * Hq * d, sizeof(double)), *lse_t = (double *)xalloc((size_t)n * Hq, sizeof(double));
    oracle_sparse_attn_tree(q + (size_t)l_ctx * Hq * d, k, v, idx_t, mask, n, l_ctx, Hq, Hkv, d, l, m, topk, scale, out_t, lse_t);
    free(q); free(k); free(v); free(dout); free(ck64); free(ckb); free(cc64); free(ccb); free(pos); free(r); free(lse_c);
    free(idx); free(margins); free(R); free(out); free(lse); free(ps); free(dq); free(dqm); free(dk); free(dkm); free(dv);
    free(dvm); free(mask); free(idx_t); free(out_t); free(lse_t);
}

int main(void) {
    /* round-trips of the bf16 helpers over specials */
    const double specials[] = {0.0, -0.0, 1.0, -1.0, 3.3895313892515355e38, 1e-45, INFINITY, -INFINITY, 65504.0, 1.0 + 1.0 / 256.0};
    for (size_t i = 0; i < sizeof specials / sizeof specials[0]; ++i) (void)oracle_bf16_to_f64(oracle_f64_to_bf16(specials[i]));
    const int32_t lens[] = {1, 31, 32, 47, 48, 64, 65, 130, 257, 333};
    for (size_t i = 0; i < sizeof lens / sizeof lens[0]; ++i) {
        run_case(lens[i], 4, 2, 3, 1, 1, 2);
        run_case(lens[i], 2, 2, 6, 1, 2, 4);
        run_case(lens[i], 8, 1, 2, 0, 0, 1);
    }
    printf("oracle_san ok\n");
    return 0;
}
