/* Walks the host side of every entry point of the C ABI -- size queries and argument validation, which
 * return before any HIP call -- in a program built with AddressSanitizer and UndefinedBehaviorSanitizer
 * against a build of the library whose host code is instrumented the same way.  No GPU is touched: every
 * call here must be rejected with an error status (or answer a size query).  Exit status 0 and
 * "abi_san ok" = clean run. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "infllmv2.h"

static int failures = 0;
#define EXPECT_ERR(call)                                                                         \
    do {                                                                                         \
        const int32_t s_ = (call);                                                               \
        if (s_ >= 0) {                                                                           \
            fprintf(stderr, "%s:%d: expected an error status, got %d\n", __FILE__, __LINE__, s_); \
            ++failures;                                                                          \
        }                                                                                        \
        (void)infllmv2_status_string(s_);                                                        \
    } while (0)

int main(void) {
    infllmv2_params good;
    memset(&good, 0, sizeof good);
    good.head_dim = 128;
    good.n_q_heads = 32;
    good.n_kv_heads = 2;
    good.block_size = 64;
    good.kernel_size = 32;
    good.kernel_stride = 16;
    good.topk = 16;
    good.n_init_blocks = 1;
    good.n_local_blocks = 2;
    good.softmax_scale = 0.088388f;
    good.lse_coarse_ratio = 1;
    infllmv2_params bad = good;
    bad.head_dim = 96;
    infllmv2_params bad_rho = good;
    bad_rho.lse_coarse_ratio = 3;
    void *fake = (void *)(uintptr_t)0x10000;      /* non-null, aligned, never dereferenced: validation fails first */
    const infllmv2_tensor t = {fake, 1 << 20, 1 << 16, 128};
    const infllmv2_tensor t_null = {NULL, 1 << 20, 1 << 16, 128};
    const infllmv2_tensor t_odd = {(void *)(uintptr_t)0x10002, 1 << 20, 1 << 16, 128};
    const int32_t *sl = (const int32_t *)fake;
    int32_t *idx = (int32_t *)fake;
    float *lse = (float *)fake;
    const uint64_t *mask = (const uint64_t *)fake;

    for (int32_t st = -8; st <= 1; ++st) (void)infllmv2_status_string(st);
    for (int32_t op = -1; op <= 12; ++op) {
        (void)infllmv2_workspace_bytes(op, &good, 1, 4096);
        (void)infllmv2_workspace_bytes(op, &good, 64, 131072);
        (void)infllmv2_workspace_bytes(op, &good, 0, 0);
        (void)infllmv2_workspace_bytes(op, &good, -1, -5);
        (void)infllmv2_workspace_bytes(op, &good, 1 << 30, 1 << 30);
        (void)infllmv2_workspace_bytes(op, &bad, 1, 4096);
        (void)infllmv2_workspace_bytes(op, NULL, 1, 4096);
        (void)infllmv2_verify_workspace_bytes(op, &good, 1, 4096, 16);
        (void)infllmv2_verify_workspace_bytes(op, &good, 1, 4096, 0);
        (void)infllmv2_verify_workspace_bytes(op, &good, 1, 4096, 65);
        (void)infllmv2_verify_workspace_bytes(op, NULL, 1, 4096, 16);
    }
    const infllmv2_params *prms[] = {NULL, &bad, &bad_rho};
    for (int i = 0; i < 3; ++i) {
        const infllmv2_params *p = prms[i];
        EXPECT_ERR(infllmv2_compress_keys(p, &t, sl, 1, 4096, 0, &t, NULL));
        EXPECT_ERR(infllmv2_select_blocks(p, INFLLMV2_MODE_PREFILL, &t, &t, sl, 1, 4096, idx, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_block_scores(p, &t, &t, sl, 1, 4096, lse, 64, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_prefill(p, &t, &t, &t, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_bwd(p, &t, &t, &t, &t, &t, lse, sl, 1, 4096, idx, &t, &t, &t, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_decode(p, &t, &t, &t, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_decode_noalloc(p, &t, &t, &t, sl, 1, 4096, idx, &t, lse, NULL));
        EXPECT_ERR(infllmv2_append_kv(p, &t, &t, &t, &t, &t, sl, 1, 4096, NULL));
        EXPECT_ERR(infllmv2_decode_step(p, &t, &t, &t, &t, &t, &t, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_append_kv_verify(p, &t, &t, &t, &t, &t, sl, 1, 4096, 8, NULL));
        EXPECT_ERR(infllmv2_select_blocks_verify(p, &t, &t, sl, 1, 4096, 8, idx, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_verify(p, &t, &t, &t, sl, 1, 4096, 8, mask, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_verify_step(p, &t, &t, &t, &t, &t, &t, sl, 1, 4096, 8, mask, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_select_blocks_shared(p, &t, &t, sl, 1, 4096, idx, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_prefill_shared(p, &t, &t, &t, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
    }
    /* good parameters, something else wrong: a null or misaligned tensor, sizes out of range, no workspace */
    const infllmv2_tensor *bad_t[] = {NULL, &t_null, &t_odd};
    for (int i = 0; i < 3; ++i) {
        const infllmv2_tensor *x = bad_t[i];
        EXPECT_ERR(infllmv2_compress_keys(&good, x, sl, 1, 4096, 0, &t, NULL));
        EXPECT_ERR(infllmv2_compress_keys(&good, &t, sl, 1, 4096, 0, x, NULL));
        EXPECT_ERR(infllmv2_select_blocks(&good, INFLLMV2_MODE_DECODE, x, &t, sl, 1, 4096, idx, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_block_scores(&good, &t, x, sl, 1, 4096, lse, 64, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_prefill(&good, &t, x, &t, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_bwd(&good, &t, &t, &t, &t, x, lse, sl, 1, 4096, idx, &t, &t, &t, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_decode(&good, &t, &t, x, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_decode_noalloc(&good, &t, &t, &t, sl, 1, 4096, idx, x, lse, NULL));
        EXPECT_ERR(infllmv2_append_kv(&good, &t, x, &t, &t, &t, sl, 1, 4096, NULL));
        EXPECT_ERR(infllmv2_decode_step(&good, &t, &t, &t, x, &t, &t, sl, 1, 4096, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_append_kv_verify(&good, x, &t, &t, &t, &t, sl, 1, 4096, 8, NULL));
        EXPECT_ERR(infllmv2_select_blocks_verify(&good, &t, x, sl, 1, 4096, 8, idx, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_verify(&good, x, &t, &t, sl, 1, 4096, 8, mask, idx, &t, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_verify_step(&good, &t, &t, &t, &t, &t, &t, sl, 1, 4096, 8, mask, idx, x, lse, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_select_blocks_shared(&good, x, &t, sl, 1, 4096, idx, fake, 1 << 30, NULL));
        EXPECT_ERR(infllmv2_sparse_attn_prefill_shared(&good, &t, &t, &t, sl, 1, 4096, idx, x, lse, fake, 1 << 30, NULL));
    }
    EXPECT_ERR(infllmv2_compress_keys(&good, &t, NULL, 1, 4096, 0, &t, NULL));
    EXPECT_ERR(infllmv2_compress_keys(&good, &t, sl, -1, 4096, 0, &t, NULL));
    EXPECT_ERR(infllmv2_compress_keys(&good, &t, sl, 1, -4096, 0, &t, NULL));
    EXPECT_ERR(infllmv2_select_blocks(&good, 7, &t, &t, sl, 1, 4096, idx, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_select_blocks(&good, INFLLMV2_MODE_PREFILL, &t, &t, sl, 1, 4096, idx, NULL, 0, NULL));
    EXPECT_ERR(infllmv2_select_blocks(&good, INFLLMV2_MODE_PREFILL, &t, &t, sl, 1, 4096, idx, fake, 16, NULL));
    EXPECT_ERR(infllmv2_select_blocks(&good, INFLLMV2_MODE_PREFILL, &t, &t, sl, 1, 4096, idx, (void *)(uintptr_t)0x10010, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_select_blocks(&good, INFLLMV2_MODE_DECODE, &t, &t, sl, 1, 1 << 30, idx, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_block_scores(&good, &t, &t, sl, 1, 4096, lse, 63, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_block_scores(&good, &t, &t, sl, 1, 4096, NULL, 64, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_prefill(&good, &t, &t, &t, sl, 1, 4096, NULL, &t, lse, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_prefill(&good, &t, &t, &t, sl, 1, 4096, idx, &t, lse, NULL, 0, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_bwd(&good, &t, &t, &t, &t, &t, NULL, sl, 1, 4096, idx, &t, &t, &t, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_bwd(&good, &t, &t, &t, &t, &t, lse, sl, 1, 4096, idx, &t, &t, &t, NULL, 0, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_decode(&good, &t, &t, &t, sl, 1, 4096, idx, &t, NULL, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_decode(&good, &t, &t, &t, sl, 1, 4096, idx, &t, lse, NULL, 0, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_decode_noalloc(&good, &t, &t, &t, sl, 4096, 4096, idx, &t, lse, NULL));   /* beyond the fixed scratch */
    EXPECT_ERR(infllmv2_decode_step(&good, &t, &t, &t, &t, &t, &t, sl, 1, 4096, idx, &t, lse, NULL, 0, NULL));
    EXPECT_ERR(infllmv2_select_blocks_verify(&good, &t, &t, sl, 1, 4096, 0, idx, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_select_blocks_verify(&good, &t, &t, sl, 1, 4096, 65, idx, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_sparse_attn_verify(&good, &t, &t, &t, sl, 1, 4096, 8, NULL, idx, &t, lse, fake, 1 << 30, NULL));
    EXPECT_ERR(infllmv2_verify_step(&good, &t, &t, &t, &t, &t, &t, sl, 1, 4096, 8, mask, idx, &t, lse, NULL, 0, NULL));
    EXPECT_ERR(infllmv2_select_blocks_shared(&good, &t, &t, sl, 1, 4096, idx, NULL, 0, NULL));
    if (failures) return 1;
    printf("abi_san ok\n");
    return 0;
}
