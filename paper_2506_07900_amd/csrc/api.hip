// C ABI of the library: argument validation (host only, before any HIP call) and dispatch to
// the kernel launchers.  See include/infllmv2.h for the contract of every entry point.
#include "common.h"

using namespace infllmv2;

namespace {

constexpr int32_t kMaxDecodeSeqlen = 262144;   // decode selection: at most 256 log-sum-exp partials per head
constexpr int32_t kMaxDraft = 64;              // one uint64 mask word per drafted token

int32_t check_params(const infllmv2_params *p) {
    if (!p) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->topk <= 0 || p->n_init_blocks < 0 ||
        p->n_local_blocks < 0 || p->head_dim <= 0 || p->block_size <= 0 || p->kernel_size <= 0 ||
        p->kernel_stride <= 0)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (!(p->softmax_scale > 0.f) || !(p->softmax_scale < 1e30f)) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->n_q_heads % p->n_kv_heads != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->topk < p->n_init_blocks + p->n_local_blocks) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->head_dim != kHeadDim || p->block_size != kBlock || p->kernel_size != kKernel ||
        p->kernel_stride != kStride)
        return INFLLMV2_ERR_UNSUPPORTED;
    const int g = p->n_q_heads / p->n_kv_heads;
    if (!(g == 1 || g == 2 || g == 4 || g == 8 || g == 16)) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->topk > kMaxTopk) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->lse_coarse_ratio < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->lse_coarse_ratio > 1) {                       // approximate log-sum-exp
        const int rho = p->lse_coarse_ratio;
        if (!(rho == 2 || rho == 4) || g != 16) return INFLLMV2_ERR_UNSUPPORTED;
        // a query that has candidate blocks must see at least one coarse kernel
        if ((p->n_init_blocks + p->n_local_blocks) * p->block_size < 2 * rho * p->kernel_stride)
            return INFLLMV2_ERR_UNSUPPORTED;
    }
    return INFLLMV2_OK;
}

int32_t check_sizes(int32_t batch, int32_t max_seqlen) {
    if (batch < 0 || max_seqlen < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (batch > 65535) return INFLLMV2_ERR_UNSUPPORTED;
    return INFLLMV2_OK;
}

// query rows of a verification step: one grid-z slot each
int32_t check_draft(int32_t batch, int32_t n_draft) {
    if (n_draft < 1) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (n_draft > kMaxDraft || (int64_t)batch * n_draft > 65535) return INFLLMV2_ERR_UNSUPPORTED;
    return INFLLMV2_OK;
}

int32_t check_tensor(const infllmv2_tensor *t) {
    if (!t || !t->ptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if ((reinterpret_cast<uintptr_t>(t->ptr) & 15u) != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (t->stride_b < 0 || t->stride_h < 0 || t->stride_t < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if ((t->stride_b % 8) || (t->stride_h % 8) || (t->stride_t % 8)) return INFLLMV2_ERR_INVALID_ARGUMENT;
    return INFLLMV2_OK;
}

Dims make_dims(const infllmv2_params *p, int32_t batch, int32_t max_seqlen, int32_t n_q = 1) {
    Dims d;
    d.Hq = p->n_q_heads;
    d.Hkv = p->n_kv_heads;
    d.G = p->n_q_heads / p->n_kv_heads;
    d.topk = p->topk;
    d.n_init = p->n_init_blocks;
    d.n_local = p->n_local_blocks;
    d.batch = batch;
    d.max_seqlen = max_seqlen;
    d.scale_log2 = p->softmax_scale * kLog2e;
    d.rho = p->lse_coarse_ratio > 1 ? p->lse_coarse_ratio : 1;
    d.n_q = n_q;
    d.shared_q = 0;
    return d;
}

Tensor make_tensor(const infllmv2_tensor *t) {
    Tensor r;
    r.ptr = reinterpret_cast<__bf16 *>(t->ptr);
    r.sb = t->stride_b;
    r.sh = t->stride_h;
    r.st = t->stride_t;
    return r;
}

int32_t hip_status(int e) { return e == 0 ? INFLLMV2_OK : INFLLMV2_ERR_HIP; }

#define RETURN_IF_ERR(x)                   \
    do {                                   \
        int32_t _s = (x);                  \
        if (_s != INFLLMV2_OK) return _s;  \
    } while (0)

}  // namespace

namespace infllmv2 {
// Host-side validation of the stage-3 decode arguments, shared by the entry points that differ only in
// where their scratch memory comes from.
int32_t validate_attn_decode(const infllmv2_params *prm, const infllmv2_tensor *q, const infllmv2_tensor *k,
                             const infllmv2_tensor *v, const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                             const int32_t *block_idx, const infllmv2_tensor *out, const float *lse, Dims *dm,
                             Tensor *tq, Tensor *tk, Tensor *tv, Tensor *tout) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(v));
    RETURN_IF_ERR(check_tensor(out));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    *dm = make_dims(prm, batch, max_seqlen);
    *tq = make_tensor(q);
    *tk = make_tensor(k);
    *tv = make_tensor(v);
    *tout = make_tensor(out);
    return INFLLMV2_OK;
}
}  // namespace infllmv2

extern "C" {

const char *infllmv2_status_string(int32_t status) {
    switch (status) {
        case INFLLMV2_OK: return "ok";
        case INFLLMV2_ERR_INVALID_ARGUMENT: return "invalid argument";
        case INFLLMV2_ERR_UNSUPPORTED: return "unsupported shape";
        case INFLLMV2_ERR_WORKSPACE: return "workspace missing or too small";
        case INFLLMV2_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

size_t infllmv2_workspace_bytes(int32_t op, const infllmv2_params *prm, int32_t batch,
                                int32_t max_seqlen) {
    if (check_params(prm) != INFLLMV2_OK || check_sizes(batch, max_seqlen) != INFLLMV2_OK) return 0;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    switch (op) {
        case INFLLMV2_OP_SELECT_PREFILL: return select_prefill_ws_bytes(dm);
        case INFLLMV2_OP_SELECT_DECODE: return max_seqlen > kMaxDecodeSeqlen ? 0 : select_decode_ws_bytes(dm);
        case INFLLMV2_OP_ATTN_PREFILL: return attn_prefill_ws_bytes(dm);
        case INFLLMV2_OP_ATTN_DECODE: return attn_decode_ws_bytes(dm);
        case INFLLMV2_OP_ATTN_BWD: return attn_bwd_ws_bytes(dm);
        case INFLLMV2_OP_SELECT_SHARED: {
            Dims ds = dm;
            ds.shared_q = 1;
            return select_prefill_ws_bytes(ds);
        }
        case INFLLMV2_OP_DECODE_STEP:
            return max_seqlen > kMaxDecodeSeqlen ? 0 : select_decode_ws_bytes(dm) + attn_decode_ws_bytes(dm);
    }
    return 0;
}

size_t infllmv2_verify_workspace_bytes(int32_t op, const infllmv2_params *prm, int32_t batch,
                                       int32_t max_seqlen, int32_t n_draft) {
    if (check_params(prm) != INFLLMV2_OK || check_sizes(batch, max_seqlen) != INFLLMV2_OK ||
        check_draft(batch, n_draft) != INFLLMV2_OK)
        return 0;
    const Dims dm = make_dims(prm, batch, max_seqlen, n_draft);
    switch (op) {
        case INFLLMV2_OP_SELECT_VERIFY: return max_seqlen > kMaxDecodeSeqlen ? 0 : select_decode_ws_bytes(dm);
        case INFLLMV2_OP_ATTN_VERIFY: return attn_decode_ws_bytes(dm);
        case INFLLMV2_OP_VERIFY_STEP:
            return max_seqlen > kMaxDecodeSeqlen ? 0 : select_decode_ws_bytes(dm) + attn_decode_ws_bytes(dm);
    }
    return 0;
}

int32_t infllmv2_compress_keys(const infllmv2_params *prm, const infllmv2_tensor *k,
                               const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                               int32_t n_new_tokens, const infllmv2_tensor *ck, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens) return INFLLMV2_ERR_INVALID_ARGUMENT;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    return hip_status(launch_compress_keys(dm, make_tensor(k), make_tensor(ck), seqlens, n_new_tokens,
                                           reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_append_kv(const infllmv2_params *prm, const infllmv2_tensor *k_new,
                           const infllmv2_tensor *v_new, const infllmv2_tensor *k,
                           const infllmv2_tensor *v, const infllmv2_tensor *ck, const int32_t *seqlens,
                           int32_t batch, int32_t max_seqlen, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(k_new));
    RETURN_IF_ERR(check_tensor(v_new));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(v));
    if (ck) RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens) return INFLLMV2_ERR_INVALID_ARGUMENT;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    Tensor ckt;
    if (ck) ckt = make_tensor(ck);
    return hip_status(launch_append_kv(dm, make_tensor(k_new), make_tensor(v_new), make_tensor(k),
                                       make_tensor(v), ck ? &ckt : nullptr, seqlens,
                                       reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_append_kv_verify(const infllmv2_params *prm, const infllmv2_tensor *k_new,
                                  const infllmv2_tensor *v_new, const infllmv2_tensor *k,
                                  const infllmv2_tensor *v, const infllmv2_tensor *ck, const int32_t *seqlens,
                                  int32_t batch, int32_t max_seqlen, int32_t n_draft, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_draft(batch, n_draft));
    RETURN_IF_ERR(check_tensor(k_new));
    RETURN_IF_ERR(check_tensor(v_new));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(v));
    if (ck) RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens) return INFLLMV2_ERR_INVALID_ARGUMENT;
    const Dims dm = make_dims(prm, batch, max_seqlen, n_draft);
    Tensor ckt;
    if (ck) ckt = make_tensor(ck);
    return hip_status(launch_append_kv(dm, make_tensor(k_new), make_tensor(v_new), make_tensor(k),
                                       make_tensor(v), ck ? &ckt : nullptr, seqlens,
                                       reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_select_blocks_verify(const infllmv2_params *prm, const infllmv2_tensor *q,
                                      const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                                      int32_t max_seqlen, int32_t n_draft, int32_t *block_idx,
                                      void *workspace, size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_draft(batch, n_draft));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens || !block_idx) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (max_seqlen > kMaxDecodeSeqlen) return INFLLMV2_ERR_UNSUPPORTED;
    const Dims dm = make_dims(prm, batch, max_seqlen, n_draft);
    const size_t need = select_decode_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_select_decode(dm, make_tensor(q), make_tensor(ck), seqlens, block_idx,
                                           workspace, reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_sparse_attn_verify(const infllmv2_params *prm, const infllmv2_tensor *q,
                                    const infllmv2_tensor *k, const infllmv2_tensor *v,
                                    const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                    int32_t n_draft, const uint64_t *tree_mask, const int32_t *block_idx,
                                    const infllmv2_tensor *out, float *lse, void *workspace,
                                    size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_draft(batch, n_draft));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(v));
    RETURN_IF_ERR(check_tensor(out));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (tree_mask && (reinterpret_cast<uintptr_t>(tree_mask) & 7u) != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    const Dims dm = make_dims(prm, batch, max_seqlen, n_draft);
    const size_t need = attn_decode_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_attn_decode(dm, make_tensor(q), make_tensor(k), make_tensor(v), seqlens,
                                         block_idx, tree_mask, make_tensor(out), lse, workspace,
                                         reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_verify_step(const infllmv2_params *prm, const infllmv2_tensor *q,
                             const infllmv2_tensor *k_new, const infllmv2_tensor *v_new,
                             const infllmv2_tensor *k, const infllmv2_tensor *v, const infllmv2_tensor *ck,
                             const int32_t *seqlens, int32_t batch, int32_t max_seqlen, int32_t n_draft,
                             const uint64_t *tree_mask, int32_t *block_idx, const infllmv2_tensor *out,
                             float *lse, void *workspace, size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_draft(batch, n_draft));
    const infllmv2_tensor *ts[7] = {q, k_new, v_new, k, v, ck, out};
    for (int i = 0; i < 7; ++i) RETURN_IF_ERR(check_tensor(ts[i]));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (tree_mask && (reinterpret_cast<uintptr_t>(tree_mask) & 7u) != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (max_seqlen > kMaxDecodeSeqlen) return INFLLMV2_ERR_UNSUPPORTED;
    const Dims dm = make_dims(prm, batch, max_seqlen, n_draft);
    const size_t sel = select_decode_ws_bytes(dm), need = sel + attn_decode_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    const AppendArgs ap = {make_tensor(k_new), make_tensor(v_new), make_tensor(k), make_tensor(v)};
    return hip_status(launch_verify_step(dm, make_tensor(q), make_tensor(ck), ap, seqlens, tree_mask, block_idx,
                                         make_tensor(out), lse, workspace, reinterpret_cast<char *>(workspace) + sel,
                                         reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_decode_step(const infllmv2_params *prm, const infllmv2_tensor *q,
                             const infllmv2_tensor *k_new, const infllmv2_tensor *v_new,
                             const infllmv2_tensor *k, const infllmv2_tensor *v, const infllmv2_tensor *ck,
                             const int32_t *seqlens, int32_t batch, int32_t max_seqlen, int32_t *block_idx,
                             const infllmv2_tensor *out, float *lse, void *workspace, size_t workspace_bytes,
                             void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    const infllmv2_tensor *ts[7] = {q, k_new, v_new, k, v, ck, out};
    for (int i = 0; i < 7; ++i) RETURN_IF_ERR(check_tensor(ts[i]));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (max_seqlen > kMaxDecodeSeqlen) return INFLLMV2_ERR_UNSUPPORTED;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    const size_t sel = select_decode_ws_bytes(dm), need = sel + attn_decode_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const AppendArgs ap = {make_tensor(k_new), make_tensor(v_new), make_tensor(k), make_tensor(v)};
    return hip_status(launch_decode_step(dm, make_tensor(q), make_tensor(ck), ap, seqlens, block_idx, make_tensor(out),
                                         lse, workspace, reinterpret_cast<char *>(workspace) + sel, st));
}

int32_t infllmv2_select_blocks(const infllmv2_params *prm, int32_t mode, const infllmv2_tensor *q,
                               const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                               int32_t max_seqlen, int32_t *block_idx, void *workspace,
                               size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    if (mode != INFLLMV2_MODE_PREFILL && mode != INFLLMV2_MODE_DECODE) return INFLLMV2_ERR_INVALID_ARGUMENT;
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens || !block_idx) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (mode == INFLLMV2_MODE_DECODE && max_seqlen > kMaxDecodeSeqlen) return INFLLMV2_ERR_UNSUPPORTED;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    const size_t need = mode == INFLLMV2_MODE_PREFILL ? select_prefill_ws_bytes(dm) : select_decode_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (mode == INFLLMV2_MODE_PREFILL)
        return hip_status(launch_select_prefill(dm, make_tensor(q), make_tensor(ck), seqlens, block_idx,
                                                workspace, st));
    return hip_status(launch_select_decode(dm, make_tensor(q), make_tensor(ck), seqlens, block_idx,
                                           workspace, st));
}

int32_t infllmv2_block_scores(const infllmv2_params *prm, const infllmv2_tensor *q, const infllmv2_tensor *ck,
                              const int32_t *seqlens, int32_t batch, int32_t max_seqlen, float *block_scores,
                              int32_t scores_pitch, void *workspace, size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens || !block_scores || scores_pitch < (max_seqlen + prm->block_size - 1) / prm->block_size)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    const size_t need = select_prefill_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_select_prefill(dm, make_tensor(q), make_tensor(ck), seqlens, nullptr, workspace,
                                            reinterpret_cast<hipStream_t>(stream), block_scores, scores_pitch));
}

int32_t infllmv2_select_blocks_shared(const infllmv2_params *prm, const infllmv2_tensor *q,
                                      const infllmv2_tensor *ck, const int32_t *seqlens, int32_t batch,
                                      int32_t max_seqlen, int32_t *block_idx, void *workspace,
                                      size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(ck));
    if (!seqlens || !block_idx) return INFLLMV2_ERR_INVALID_ARGUMENT;
    Dims dm = make_dims(prm, batch, max_seqlen);
    dm.shared_q = 1;
    const size_t need = select_prefill_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_select_prefill(dm, make_tensor(q), make_tensor(ck), seqlens, block_idx, workspace,
                                            reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_sparse_attn_prefill(const infllmv2_params *prm, const infllmv2_tensor *q,
                                     const infllmv2_tensor *k, const infllmv2_tensor *v,
                                     const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                     const int32_t *block_idx, const infllmv2_tensor *out, float *lse,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(v));
    RETURN_IF_ERR(check_tensor(out));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    const size_t need = attn_prefill_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_attn_prefill(dm, make_tensor(q), make_tensor(k), make_tensor(v), seqlens,
                                          block_idx, make_tensor(out), lse, workspace,
                                          reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_sparse_attn_prefill_shared(const infllmv2_params *prm, const infllmv2_tensor *q,
                                            const infllmv2_tensor *k, const infllmv2_tensor *v,
                                            const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                            const int32_t *block_idx, const infllmv2_tensor *out, float *lse,
                                            void *workspace, size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    RETURN_IF_ERR(check_tensor(q));
    RETURN_IF_ERR(check_tensor(k));
    RETURN_IF_ERR(check_tensor(v));
    RETURN_IF_ERR(check_tensor(out));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    Dims dm = make_dims(prm, batch, max_seqlen);
    dm.shared_q = 1;
    const size_t need = attn_prefill_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_attn_prefill(dm, make_tensor(q), make_tensor(k), make_tensor(v), seqlens,
                                          block_idx, make_tensor(out), lse, workspace,
                                          reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_sparse_attn_bwd(const infllmv2_params *prm, const infllmv2_tensor *q,
                                 const infllmv2_tensor *k, const infllmv2_tensor *v,
                                 const infllmv2_tensor *out, const infllmv2_tensor *dout, const float *lse,
                                 const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                 const int32_t *block_idx, const infllmv2_tensor *dq,
                                 const infllmv2_tensor *dk, const infllmv2_tensor *dv, void *workspace,
                                 size_t workspace_bytes, void *stream) {
    RETURN_IF_ERR(check_params(prm));
    RETURN_IF_ERR(check_sizes(batch, max_seqlen));
    const infllmv2_tensor *ts[8] = {q, k, v, out, dout, dq, dk, dv};
    for (int i = 0; i < 8; ++i) RETURN_IF_ERR(check_tensor(ts[i]));
    if (!seqlens || !block_idx || !lse) return INFLLMV2_ERR_INVALID_ARGUMENT;
    // the dk/dv kernel addresses the heads of a group with 32-bit element offsets from the group's first head
    const int64_t head_span = (int64_t)(prm->n_q_heads / prm->n_kv_heads) * (q->stride_h > dout->stride_h ? q->stride_h : dout->stride_h);
    if (head_span > (int64_t)1 << 30) return INFLLMV2_ERR_UNSUPPORTED;
    const Dims dm = make_dims(prm, batch, max_seqlen);
    const size_t need = attn_bwd_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_attn_bwd(dm, make_tensor(q), make_tensor(k), make_tensor(v), make_tensor(out),
                                      make_tensor(dout), lse, seqlens, block_idx, make_tensor(dq), make_tensor(dk),
                                      make_tensor(dv), workspace, reinterpret_cast<hipStream_t>(stream)));
}

int32_t infllmv2_sparse_attn_decode(const infllmv2_params *prm, const infllmv2_tensor *q,
                                    const infllmv2_tensor *k, const infllmv2_tensor *v,
                                    const int32_t *seqlens, int32_t batch, int32_t max_seqlen,
                                    const int32_t *block_idx, const infllmv2_tensor *out, float *lse,
                                    void *workspace, size_t workspace_bytes, void *stream) {
    Dims dm;
    Tensor tq, tk, tv, tout;
    RETURN_IF_ERR(validate_attn_decode(prm, q, k, v, seqlens, batch, max_seqlen, block_idx, out, lse, &dm, &tq, &tk,
                                       &tv, &tout));
    const size_t need = attn_decode_ws_bytes(dm);
    if (need > 0 && (!workspace || workspace_bytes < need ||
                     (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0))
        return INFLLMV2_ERR_WORKSPACE;
    return hip_status(launch_attn_decode(dm, tq, tk, tv, seqlens, block_idx, nullptr, tout, lse, workspace,
                                         reinterpret_cast<hipStream_t>(stream)));
}

}  // extern "C"
