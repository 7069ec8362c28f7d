/*
 * infllmv2.h -- C ABI of the MI355X (gfx950) implementation of InfLLM v2
 * trainable block-sparse attention (MiniCPM4 report, section 2.1).
 *
 * The path has three stages (section 2.1.1, "two stages" plus the compression the
 * first one needs):
 *   1. infllmv2_compress_keys       mean-pool the keys into overlapping semantic kernels
 *   2. infllmv2_select_blocks       relevance of every key-value block to each query token,
 *                                   shared by the query heads of a group; top-k blocks plus
 *                                   the always-selected initial and local-window blocks
 *   3. infllmv2_sparse_attn_prefill / infllmv2_sparse_attn_decode
 *                                   exact softmax attention over the selected blocks only
 * plus infllmv2_append_kv, the cache append that opens a decode step, and infllmv2_decode_step, the
 * whole decode step in one call.  Built on top of the path: the approximate log-sum-exp of stage 2
 * (infllmv2_params.lse_coarse_ratio), infllmv2_sparse_attn_bwd (the gradients of stage 3), the
 * *_verify variants of the decode step for the n drafted tokens of speculative decoding (section
 * 4.1), and, as a labelled comparison that is NOT the report's method, the *_shared variants with
 * one block set per query block.
 *
 * Conventions for every entry point
 *   - Returns 0 (INFLLMV2_OK) or a negative INFLLMV2_ERR_* code; never throws, never
 *     allocates or frees device memory, never synchronises the stream.  Arguments are
 *     validated on the host before the first HIP call; on a validation error nothing
 *     is launched.
 *   - Every data pointer is a DEVICE pointer owned by the caller; `prm` and the tensor
 *     descriptors are HOST structs read during the call only.  `stream` is a hipStream_t
 *     passed as void* (NULL = the default stream).  Work is enqueued on that stream.
 *   - bf16 tensors are described by infllmv2_tensor: strides are in ELEMENTS, the
 *     head_dim axis is contiguous (stride 1) and every row must be 16-byte aligned
 *     (pointer and strides multiples of 8 elements).
 *       key / value cache, compressed keys:  element (b, h, t, c) at
 *           ptr + b*stride_b + h*stride_h + t*stride_t + c        h = key-value head
 *       queries, outputs:                    element (b, t, hq, c) at
 *           ptr + b*stride_b + t*stride_t + hq*stride_h + c       hq = query head
 *     Query head hq belongs to key-value head hq / G, G = n_q_heads / n_kv_heads.
 *   - `seqlens` is a device int32 [batch] array: the number of valid cache rows of each
 *     sequence.  `max_seqlen` is a host upper bound on its entries, used to size
 *     launches and buffers; entries above it are clamped to it.
 *   - Positions, blocks and semantic kernels are 0-based.  With m = block_size,
 *     p = kernel_size, s = kernel_stride:
 *       a sequence of l tokens has n_c(l) = floor((l-p)/s)+1 complete kernels (0 if l<p);
 *       query position i ranks blocks 0..floor(i/m) and sees kernels jh < n_c(i+1).
 *   - Supported shapes: head_dim 128, block_size 64, kernel_size 32, kernel_stride 16,
 *     G in {1,2,4,8,16}, topk in [max(1, n_init_blocks + n_local_blocks), 64].  Anything
 *     else returns INFLLMV2_ERR_UNSUPPORTED.
 *   - Calls that share a workspace must be ordered on one stream.
 */
#ifndef INFLLMV2_H
#define INFLLMV2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define INFLLMV2_OK 0
#define INFLLMV2_ERR_INVALID_ARGUMENT (-1) /* null pointer, bad size, bad stride or alignment  */
#define INFLLMV2_ERR_UNSUPPORTED (-2)      /* a shape outside the supported set above           */
#define INFLLMV2_ERR_WORKSPACE (-3)        /* workspace missing or smaller than the size query */
#define INFLLMV2_ERR_HIP (-4)              /* a HIP launch reported an error                   */

/* Stage selector for infllmv2_workspace_bytes. */
#define INFLLMV2_OP_SELECT_PREFILL 1
#define INFLLMV2_OP_SELECT_DECODE 2
#define INFLLMV2_OP_ATTN_PREFILL 3
#define INFLLMV2_OP_ATTN_DECODE 4
#define INFLLMV2_OP_ATTN_BWD 7
#define INFLLMV2_OP_DECODE_STEP 8
#define INFLLMV2_OP_SELECT_SHARED 9
/* Stage selector for infllmv2_verify_workspace_bytes. */
#define INFLLMV2_OP_SELECT_VERIFY 5
#define INFLLMV2_OP_ATTN_VERIFY 6
#define INFLLMV2_OP_VERIFY_STEP 10

/* Query layout selector for infllmv2_select_blocks. */
#define INFLLMV2_MODE_PREFILL 0 /* one query per cached token: query t sits at position t        */
#define INFLLMV2_MODE_DECODE 1  /* one query per sequence, at position seqlens[b]-1              */

/* Hyper-parameters of section 2.1 ("Hyper-Parameter Recommendation": p = 32, s = 16). */
typedef struct infllmv2_params {
    int32_t head_dim;        /* d, 128                                                         */
    int32_t n_q_heads;       /* Hq                                                             */
    int32_t n_kv_heads;      /* Hkv                                                            */
    int32_t block_size;      /* m, tokens per key-value block, 64                              */
    int32_t kernel_size;     /* p, tokens per semantic kernel, 32                              */
    int32_t kernel_stride;   /* s, stride between semantic kernels, 16                         */
    int32_t topk;            /* k, blocks attended per query token INCLUDING the forced ones   */
    int32_t n_init_blocks;   /* leading blocks whose relevance is set to infinity              */
    int32_t n_local_blocks;  /* trailing blocks (the query's own and the ones before it) forced */
    float softmax_scale;     /* multiplies q.k in both the relevance softmax and the attention */
    int32_t lse_coarse_ratio; /* rho = s_c / s of the approximate log-sum-exp of the relevance softmax
                                ("Efficient Top-K Implementation", last paragraph); 0 or 1 = exact.
                                rho = 2 or 4 needs G = 16 and
                                (n_init_blocks + n_local_blocks) * m >= 2 * rho * s (other group sizes
                                return INFLLMV2_ERR_UNSUPPORTED: the coarse pass exists in the kernels
                                specialised for G = 16, the group size of "Hyper-Parameter
                                Recommendation", only; every other G runs the exact two passes, of which
                                this is an optimisation).  A coarse kernel is
                                the bf16-rounded mean of the rho disjoint semantic kernels
                                rho*c, rho*c+2, .., that tile tokens [rho*s*c, rho*s*(c+2)); the
                                softmax denominator of a query head becomes
                                rho * sum over visible coarse kernels of exp(scale q.CKc), and relevance
                                scores are clamped to [2^-100, 2^100].  It changes which blocks win. */
} infllmv2_params;

/* A bf16 device tensor with a contiguous head_dim axis; strides in elements (see above). */
typedef struct infllmv2_tensor {
    void *ptr;
    int64_t stride_b;
    int64_t stride_h;
    int64_t stride_t;
} infllmv2_tensor;

/* Human-readable name of a status code (static storage). */
const char *infllmv2_status_string(int32_t status);

/* Bytes of device scratch the given stage needs for `batch` sequences of at most `max_seqlen`
 * cached tokens (0 if the stage needs none, or if the arguments are invalid). */
size_t infllmv2_workspace_bytes(int32_t op, const infllmv2_params *prm, int32_t batch,
                                int32_t max_seqlen);

/*
 * Stage 1 -- semantic-kernel representations (section 2.1.2, "Semantic Kernels"):
 *     ck[b, h, jh, :] = Mean(k[b, h, jh*s : jh*s+p, :]),   jh < n_c(seqlens[b]),
 * accumulated in fp64 in token order and rounded once to bf16 (ties to even).
 *   k             in   bf16 cache [batch, Hkv, >=max_seqlen, d]
 *   ck            out  bf16 [batch, Hkv, >=n_c(max_seqlen), d]; stride_t is the kernel stride
 *   n_new_tokens  <= 0: write every kernel of every sequence.
 *                 >  0: incremental update -- write only the kernels completed by the last
 *                       n_new_tokens tokens, i.e. jh in [n_c(seqlens[b]-n_new_tokens), n_c(seqlens[b]));
 *                       rows written earlier are left untouched, so after any sequence of
 *                       appends ck equals the from-scratch result bit for bit.
 * Rows jh >= n_c(seqlens[b]) are never written.
 */
int32_t infllmv2_compress_keys(const infllmv2_params *prm, const infllmv2_tensor *k,
                               const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                               int32_t n_new_tokens, const infllmv2_tensor *ck, void *stream);

/*
 * Stage 2 -- block selection (section 2.1.2, "Dynamic Contextual Block Selection", Eq. 1,
 * "Top-K Blocks Sharing", "Efficient Top-K Implementation").  For every key-value head h and
 * query token at position i:
 *     z_g[jh] = softmax_scale * <q_g, ck[h, jh]>              g in the group of h, jh < n_c(i+1)
 *     r[jh]   = max( mean_g softmax_jh(z_g)[jh], 2^-100 )     (softmax first, then the group mean)
 *     R[j]    = max of r[jh] over kernels whose tokens intersect block j,   j <= floor(i/m)
 *     R[j]    = +inf for j < n_init_blocks and for j > floor(i/m) - n_local_blocks
 *     select the min(topk, floor(i/m)+1) blocks of largest R, ties to the lower index.
 * The softmax is computed exactly in two passes (log-sum-exp first, scores second).
 *   mode       INFLLMV2_MODE_PREFILL: q is [batch, max_seqlen, Hq, d], row t = position t,
 *              rows t >= seqlens[b] are ignored; n_q = max_seqlen rows per sequence.
 *              INFLLMV2_MODE_DECODE: q is [batch, 1, Hq, d], position seqlens[b]-1; n_q = 1.
 *   ck         in   compressed keys with at least n_c(seqlens[b]) valid rows per sequence
 *   block_idx  out  int32 [batch, Hkv, n_q, topk] contiguous: selected block indices in
 *              ascending order, padded with -1.  Prefill rows t >= seqlens[b] are not written.
 *   workspace  device scratch of infllmv2_workspace_bytes(INFLLMV2_OP_SELECT_*, ...) bytes,
 *              256-byte aligned; contents are undefined before and after the call.  Prefill: the
 *              log-sum-exps of pass 1 (4 bytes per query token and head) and a tiled copy of ck, so
 *              linear in max_seqlen; the block scores are ranked inside pass 2, chunk by chunk in
 *              on-chip memory, and are never stored.
 */
int32_t infllmv2_select_blocks(const infllmv2_params *prm, int32_t mode, const infllmv2_tensor *q,
                               const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                               int32_t max_seqlen, int32_t *block_idx, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * The block scores stage 2 ranks, for inspection and for checking the selection's arithmetic (not a
 * step of the method: infllmv2_select_blocks ranks the same scores on chip and never stores them).
 * Prefill queries only.  For every key-value head h, query token t < seqlens[b] and candidate block j
 * (n_init_blocks <= j <= floor(t/m) - n_local_blocks):
 *     block_scores[((b * Hkv + h) * max_seqlen + t) * scores_pitch + j] = R[j]   of Eq. 1 as stated above,
 * fp32, -inf when no semantic kernel that intersects block j is visible to the query.  Entries of
 * other blocks and of rows t >= seqlens[b] may or may not be written.
 *   block_scores  out  fp32 device buffer of batch * Hkv * max_seqlen * scores_pitch elements
 *   scores_pitch       row pitch in elements, >= ceil(max_seqlen / m)
 *   workspace          as for infllmv2_select_blocks in prefill mode (INFLLMV2_OP_SELECT_PREFILL)
 */
int32_t infllmv2_block_scores(const infllmv2_params *prm, const infllmv2_tensor *q,
                              const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                              int32_t max_seqlen, float *block_scores, int32_t scores_pitch,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Stage 3, prefill -- attention over the selected blocks (section 2.1.1, second stage):
 *     T_i = { t <= i : floor(t/m) in block_idx[b, h, i, :] }
 *     out[b, i, hq, :] = sum_{t in T_i} softmax_t(softmax_scale * <q_i, k_t>) v_t
 *     lse[b, i, hq]    = log sum_{t in T_i} exp(softmax_scale * <q_i, k_t>)      (natural log)
 * bf16 products accumulated in fp32; probabilities are rounded to bf16 before the value
 * product, their fp32 sum is taken before rounding.
 *   q, out     [batch, max_seqlen, Hq, d] bf16 (rows t >= seqlens[b] ignored / not written)
 *   k, v       bf16 caches [batch, Hkv, >=max_seqlen, d]
 *   block_idx  in   int32 [batch, Hkv, max_seqlen, topk]; entries < 0 or > floor(i/m) are skipped;
 *              each row must be duplicate-free
 *   lse        out  fp32 [batch, max_seqlen, Hq] contiguous
 *   workspace  device scratch of infllmv2_workspace_bytes(INFLLMV2_OP_ATTN_PREFILL, ...) bytes
 *              (a re-laid-out copy of the K and V blocks: 32 KiB per block and key-value head)
 */
int32_t infllmv2_sparse_attn_prefill(const infllmv2_params *prm, const infllmv2_tensor *q,
                                     const infllmv2_tensor *k, const infllmv2_tensor *v,
                                     const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                     const int32_t *block_idx, const infllmv2_tensor *out,
                                     float *lse, void *workspace, size_t workspace_bytes,
                                     void *stream);

/*
 * Stage 3, backward -- gradients of infllmv2_sparse_attn_prefill's output with respect to q, k and v
 * for an upstream gradient dout, the block sets held fixed (section 2.1: the sparse attention is
 * trainable; the selection is a discrete choice and the mean-pooled semantic kernels have no
 * parameters, so nothing flows through stage 2).  With p = exp(softmax_scale <q_i, k_t> - lse) over
 * T_i and D = <dout_i, out_i> per (token, head):
 *     dv_t = sum p dout_i        ds = p (<dout_i, v_t> - D)
 *     dq_i = softmax_scale sum_t ds k_t        dk_t = softmax_scale sum ds q_i
 * (sums for dk, dv over the tokens that selected t's block and the query heads of the group).
 * bf16 products accumulated in fp32; p and ds are rounded to bf16 before the second products;
 * dk, dv are merged with fp32 atomic adds (the last bits depend on the order).
 *   q, out, dout  in   [batch, max_seqlen, Hq, d] bf16: the forward's input, output and its gradient
 *                      (q, dout: group size x head stride at most 2^30 elements, else INFLLMV2_ERR_UNSUPPORTED)
 *   k, v          in   bf16 caches [batch, Hkv, >=max_seqlen, d]
 *   lse           in   fp32 [batch, max_seqlen, Hq], the forward's log-sum-exp
 *   block_idx     in   int32 [batch, Hkv, max_seqlen, topk], as given to the forward
 *   dq            out  [batch, max_seqlen, Hq, d] bf16 (rows t >= seqlens[b] not written)
 *   dk, dv        out  [batch, Hkv, >=max_seqlen, d] bf16 (rows t >= seqlens[b] not written)
 *   workspace     device scratch of infllmv2_workspace_bytes(INFLLMV2_OP_ATTN_BWD, ...) bytes: packed
 *                 copies of the K and V blocks, D and the exponent offsets per (token, head), a block x token
 *                 membership bitmap, fp32 dk / dv
 */
int32_t infllmv2_sparse_attn_bwd(const infllmv2_params *prm, const infllmv2_tensor *q,
                                 const infllmv2_tensor *k, const infllmv2_tensor *v,
                                 const infllmv2_tensor *out, const infllmv2_tensor *dout, const float *lse,
                                 const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                 const int32_t *block_idx, const infllmv2_tensor *dq,
                                 const infllmv2_tensor *dk, const infllmv2_tensor *dv, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * Stage 3, decode -- the same attention for the single query at position seqlens[b]-1
 * (section 2.1.3, "Different Granularity for Query and Key-Value Tokens": token-level
 * queries are what makes the method usable in decoding).
 *   q, out     [batch, 1, Hq, d] bf16
 *   k, v       bf16 caches [batch, Hkv, >=max_seqlen, d]
 *   block_idx  in   int32 [batch, Hkv, 1, topk]
 *   lse        out  fp32 [batch, Hq]
 *   workspace  device scratch of infllmv2_workspace_bytes(INFLLMV2_OP_ATTN_DECODE, ...) bytes
 */
int32_t infllmv2_sparse_attn_decode(const infllmv2_params *prm, const infllmv2_tensor *q,
                                    const infllmv2_tensor *k, const infllmv2_tensor *v,
                                    const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                    const int32_t *block_idx, const infllmv2_tensor *out,
                                    float *lse, void *workspace, size_t workspace_bytes,
                                    void *stream);

/*
 * infllmv2_sparse_attn_decode for callers that cannot allocate device memory or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus
 * the workspace, same kernels, same out and lse bit for bit.  The per-block partial results live in a
 * fixed array of INFLLMV2_NOALLOC_SCRATCH_BYTES in device memory that belongs to the library's code
 * object: every GPU the library runs on holds its own copy until the process ends, looked up on the
 * first call made with that GPU current (`stream` must belong to the current device).
 *   Limit: batch * n_q_heads * topk * 520 bytes (rounded up to 256-byte multiples per array) must fit the
 *   array, e.g. batch 7 at 32 query heads and top-k 32; beyond it INFLLMV2_ERR_UNSUPPORTED is returned
 *   and nothing is launched.
 *   All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *   different threads) race on it and must be ordered by the caller.  Nothing needs clearing between
 *   calls: every partial a call reads is written by that call first.
 * Calls no hipMalloc / hipFree, directly or through a library.
 */
#define INFLLMV2_NOALLOC_SCRATCH_BYTES (4u << 20)
int32_t infllmv2_sparse_attn_decode_noalloc(const infllmv2_params *prm, const infllmv2_tensor *q,
                                            const infllmv2_tensor *k, const infllmv2_tensor *v,
                                            const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                            const int32_t *block_idx, const infllmv2_tensor *out,
                                            float *lse, void *stream);

/*
 * Decode-step cache append: writes the new token's key and value rows at position
 * seqlens[b]-1 of each sequence's cache (seqlens already counts the new token).
 *   k_new, v_new  in   bf16 [batch, Hkv, 1, d]  (stride_t unused)
 *   k, v          out  bf16 caches [batch, Hkv, >=max_seqlen, d]
 *   ck            out  optional (NULL to skip): the compressed-key cache of
 *                      infllmv2_compress_keys.  When the new token completes a semantic kernel
 *                      (seqlens[b] >= p and seqlens[b]-p a multiple of s) its representation is
 *                      written in the same launch, bit-identical to what
 *                      infllmv2_compress_keys(n_new_tokens = 1) writes after the append
 *                      (section 5.4: per decode step only the semantic-kernel representations grow).
 * Sequences with seqlens[b] < 1 are skipped.
 */
int32_t infllmv2_append_kv(const infllmv2_params *prm, const infllmv2_tensor *k_new,
                           const infllmv2_tensor *v_new, const infllmv2_tensor *k,
                           const infllmv2_tensor *v, const infllmv2_tensor *ck,
                           const int32_t *seqlens, int32_t batch, int32_t max_seqlen, void *stream);

/*
 * One decode step in one call (section 5.4: per step only the semantic-kernel representations grow):
 * infllmv2_append_kv (with ck) + infllmv2_select_blocks(INFLLMV2_MODE_DECODE) +
 * infllmv2_sparse_attn_decode, with the append folded into the first selection kernel and the top-k
 * into the per-block attention kernel: four launches instead of six (five when batch * Hkv * topk
 * exceeds 1024: the top-k then runs once per row in a launch of its own), the same caches, ck,
 * block_idx, out and lse bit for bit.
 *   q, out        [batch, 1, Hq, d] bf16;  k_new, v_new  [batch, Hkv, 1, d] bf16
 *   k, v, ck      the caches (updated in place);  seqlens counts the new token
 *   block_idx     out  int32 [batch, Hkv, 1, topk];  lse  out  fp32 [batch, Hq]
 *   workspace     infllmv2_workspace_bytes(INFLLMV2_OP_DECODE_STEP, ...) bytes
 */
int32_t infllmv2_decode_step(const infllmv2_params *prm, const infllmv2_tensor *q,
                             const infllmv2_tensor *k_new, const infllmv2_tensor *v_new,
                             const infllmv2_tensor *k, const infllmv2_tensor *v, const infllmv2_tensor *ck,
                             const int32_t *seqlens, int32_t batch, int32_t max_seqlen, int32_t *block_idx,
                             const infllmv2_tensor *out, float *lse, void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * Draft verification (section 4.1, "InfLLM v2 for Target Model": the target model checks n drafted
 * tokens in one step; inside the last n x n region of the attention the causal triangle is replaced
 * by a tree mask, bit-packed in uint64).  The three calls below are the decode step for n_draft
 * query tokens per sequence, 1 <= n_draft <= 64, batch * n_draft <= 65535:
 *   - the drafted tokens occupy the LAST n_draft cache rows of each sequence, in draft order:
 *     draft token t sits at position seqlens[b] - n_draft + t (seqlens counts them);
 *   - draft token t selects blocks exactly as a query at that position does in
 *     infllmv2_select_blocks (the selection does not look at the tree);
 *   - it attends, inside its selected blocks, every context token (position < seqlens[b] - n_draft)
 *     and draft token j iff bit j of tree_mask[b * n_draft + t] is set (j may exceed t only inside
 *     selected blocks; bits >= n_draft are ignored).  tree_mask == NULL means the causal chain
 *     (bit j set iff j <= t), which makes the step equal to n_draft prefill rows.
 *   A sequence with seqlens[b] < n_draft is skipped as a whole: block_idx -1, out 0, lse -inf,
 *   nothing appended.  A query whose mask hides every key of its selected blocks gets out 0, lse -inf.
 *
 * infllmv2_append_kv_verify     k_new, v_new bf16 [batch, Hkv, n_draft, d] -> cache rows
 *                               seqlens[b]-n_draft .. seqlens[b]-1; with ck != NULL the same launch
 *                               writes the semantic kernels those rows complete (the bits
 *                               infllmv2_compress_keys with n_new_tokens = n_draft writes afterwards).
 * infllmv2_select_blocks_verify q bf16 [batch, n_draft, Hq, d]; block_idx out int32
 *                               [batch, Hkv, n_draft, topk], ascending, padded with -1.
 * infllmv2_sparse_attn_verify   q, out bf16 [batch, n_draft, Hq, d]; tree_mask DEVICE uint64
 *                               [batch, n_draft] or NULL; lse out fp32 [batch, n_draft, Hq];
 *                               arithmetic as in infllmv2_sparse_attn_decode.
 * infllmv2_verify_step          the three calls in one (ck required), five launches instead of six
 *                               (the top-k is folded into the per-block attention kernel unless
 *                               batch * n_draft * Hkv * topk exceeds 1024); the same caches, ck,
 *                               block_idx, out and lse bit for bit.
 * Workspaces: infllmv2_verify_workspace_bytes(INFLLMV2_OP_SELECT_VERIFY / _ATTN_VERIFY /
 * _VERIFY_STEP, ...) (0 if the arguments are invalid), 256-byte aligned.
 */
size_t infllmv2_verify_workspace_bytes(int32_t op, const infllmv2_params *prm, int32_t batch,
                                       int32_t max_seqlen, int32_t n_draft);
int32_t infllmv2_append_kv_verify(const infllmv2_params *prm, const infllmv2_tensor *k_new,
                                  const infllmv2_tensor *v_new, const infllmv2_tensor *k,
                                  const infllmv2_tensor *v, const infllmv2_tensor *ck,
                                  const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                  int32_t n_draft, void *stream);
int32_t infllmv2_select_blocks_verify(const infllmv2_params *prm, const infllmv2_tensor *q,
                                      const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                                      int32_t max_seqlen, int32_t n_draft, int32_t *block_idx,
                                      void *workspace, size_t workspace_bytes, void *stream);
int32_t infllmv2_sparse_attn_verify(const infllmv2_params *prm, const infllmv2_tensor *q,
                                    const infllmv2_tensor *k, const infllmv2_tensor *v,
                                    const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                    int32_t n_draft, const uint64_t *tree_mask, const int32_t *block_idx,
                                    const infllmv2_tensor *out, float *lse, void *workspace,
                                    size_t workspace_bytes, void *stream);
int32_t infllmv2_verify_step(const infllmv2_params *prm, const infllmv2_tensor *q,
                             const infllmv2_tensor *k_new, const infllmv2_tensor *v_new,
                             const infllmv2_tensor *k, const infllmv2_tensor *v, const infllmv2_tensor *ck,
                             const int32_t *seqlens, int32_t batch, int32_t max_seqlen, int32_t n_draft,
                             const uint64_t *tree_mask, int32_t *block_idx, const infllmv2_tensor *out,
                             float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Query-block-shared selection -- a COMPARISON VARIANT, not the report's method (section 2.1.3 argues
 * for token-level queries; infllmv2_select_blocks is the method).  The m = 64 tokens of query block I
 * attend one common block set: block j is scored by the mean over the tokens of I of their per-token
 * block relevance R[j] (as in infllmv2_select_blocks), the first n_init_blocks blocks and the last
 * n_local_blocks blocks up to I are forced, the min(topk, I+1) best are taken, ties to the lower index.
 *   q          [batch, max_seqlen, Hq, d]
 *   block_idx  out  int32 [batch, Hkv, ceil(max_seqlen/64), topk], ascending, padded with -1; rows of
 *              query blocks that start at or after seqlens[b] are not written
 *   workspace  infllmv2_workspace_bytes(INFLLMV2_OP_SELECT_SHARED, ...) bytes
 */
int32_t infllmv2_select_blocks_shared(const infllmv2_params *prm, const infllmv2_tensor *q,
                                      const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                                      int32_t max_seqlen, int32_t *block_idx, void *workspace,
                                      size_t workspace_bytes, void *stream);

/*
 * The attention for block sets shared by the 64 tokens of a query block (the same COMPARISON VARIANT):
 * out and lse as infllmv2_sparse_attn_prefill computes them when every token of query block I is given
 * row I of block_idx.
 *   block_idx  in   int32 [batch, Hkv, ceil(max_seqlen/64), topk]; entries < 0 or > I are skipped; each
 *              row must be duplicate-free
 *   workspace  infllmv2_workspace_bytes(INFLLMV2_OP_ATTN_PREFILL, ...) bytes
 */
int32_t infllmv2_sparse_attn_prefill_shared(const infllmv2_params *prm, const infllmv2_tensor *q,
                                            const infllmv2_tensor *k, const infllmv2_tensor *v,
                                            const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                            const int32_t *block_idx, const infllmv2_tensor *out, float *lse,
                                            void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* INFLLMV2_H */
