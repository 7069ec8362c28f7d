/*
 * CPU oracle for InfLLM v2 block-sparse attention (MiniCPM4 report, section 2.1).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code with the HIP path, and the
 * product never calls it: only the tests, the smoke check and the cpu_baseline
 * leg of the benchmark may load it.
 *
 * Everything is fp64 computed from bf16-valued inputs (bf16 bit patterns in
 * uint16 arrays).  One sequence per call; rows are independent, so the only
 * parallelism is an OpenMP `parallel for` over query rows.  There is no tiling,
 * fusion or reordering: each function is the formula written out.
 *
 * Notation follows section 2.1: l sequence length, m block size, p / s semantic
 * kernel size / stride, k number of selected blocks, G = Hq / Hkv query heads per
 * key-value head, d head dimension.  Positions, blocks and kernels are 0-based.
 *
 * Readings taken where the text is silent (each is a definition shared with the
 * HIP path, none can be pinned to a printed example -- "parity unpinned" for the
 * readings themselves; the arithmetic of every function below IS pinned by the
 * CPU tests):
 *   - only complete semantic kernels exist:  n_c(l) = floor((l-p)/s)+1  (0 if l<p);
 *   - query i sees kernel jh iff the kernel lies wholly at or before i:
 *     jh*s + p - 1 <= i, i.e. n_vis(i) = n_c(i+1);
 *   - the softmax over kernels uses the attention scale;
 *   - group score = mean over the G heads of the per-head softmax;
 *   - scores are floored at 2^-100 so that underflow gives deterministic ties;
 *   - ties go to the lower block index;
 *   - query i ranks blocks 0..floor(i/m); the last one may be partial;
 *   - forced blocks: the first n_init blocks and the last n_local blocks up to
 *     and including the query's own.
 * Readings for the approximate log-sum-exp ("Efficient Top-K Implementation", last
 * paragraph; the report gives no formula, so all of this is a definition -- parity
 * unpinned for the reading, the arithmetic is pinned):
 *   - a coarse semantic kernel covers s_c = rho*s tokens of stride and 2*s_c tokens of
 *     size (the same overlap as p = 2s); it is the mean of the rho disjoint fine kernels
 *     that tile its window, taken from the bf16 fine representations and rounded to bf16;
 *   - a query sees a coarse kernel iff it sees all of its fine kernels;
 *   - LSE_approx = log sum_{visible coarse} exp(scale <q, CKc>) + log(rho)   (there are
 *     rho times fewer coarse kernels); 0 when no coarse kernel is visible (no selection
 *     depends on it when (n_init + n_local) * m >= 2 * s_c);
 *   - scores exp(z - LSE_approx) are no longer bounded by 1: they are clamped above at 2^100.
 * Reading for the backward pass (section 2.1 calls the attention trainable and gives no backward
 * formulas -- parity unpinned for the reading, the arithmetic is pinned against automatic
 * differentiation): gradients flow to q, k, v through the stage-3 attention only, block sets fixed.
 * Reading for tree-style draft verification (section 4.1, "InfLLM v2 for Target Model"; the
 * report says only that the local mask of the last n x n region is bit-packed in uint64 --
 * parity unpinned for the reading, the arithmetic is pinned):
 *   - the n <= 64 drafted tokens are already in the cache at positions l_ctx .. l_ctx+n-1 in
 *     draft order; draft token t selects blocks as a query at position l_ctx+t would (the
 *     selection does not look at the tree); only the attention's causal test inside the last
 *     n x n region is replaced by "bit j of tree_mask[t]".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_SCORE_FLOOR 7.888609052210118e-31 /* 2^-100 */
#define ORACLE_SCORE_CEIL 1.2676506002282294e30  /* 2^100, approximate-LSE mode only */

/* ---- bf16 helpers -------------------------------------------------------- */

static double bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round an fp64 value straight to bf16 (8 significant bits), ties to even.
 * Rounding goes directly from fp64 so there is no double rounding through fp32. */
static uint16_t f64_to_bf16(double x) {
    float f;
    uint32_t u;
    if (isnan(x)) return 0x7fc0;
    if (x == 0.0 || isinf(x)) {
        f = (float)x;
    } else {
        int e = ilogb(x);
        if (e < -126) e = -126;              /* subnormal range: fixed quantum   */
        double q = ldexp(1.0, e - 7);        /* value of the last kept bit        */
        double r = rint(x / q) * q;          /* rint: round-half-even by default  */
        f = (float)r;                        /* exact, or overflows to +-inf      */
    }
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

/* ---- counts -------------------------------------------------------------- */

/* Number of complete semantic kernels in a sequence of l tokens (section 2.1.2,
 * "Semantic Kernels": windows K[jh*s : jh*s+p]). */
int32_t oracle_num_kernels(int32_t l, int32_t p, int32_t s) {
    if (l < p) return 0;
    return (l - p) / s + 1;
}

/* ---- O1: mean-pool compression ------------------------------------------- */

/* CK[h, jh, :] = Mean(K[h, jh*s : jh*s+p, :])   (section 2.1.2, the Mean(.) in the
 * definition of r_kernel).
 *   k_bits   [Hkv, l, d]  bf16 bit patterns
 *   ck_f64   [Hkv, n_c, d] unrounded means (may be NULL)
 *   ck_bits  [Hkv, n_c, d] means rounded to bf16, ties to even (may be NULL)
 * Returns n_c. */
int32_t oracle_compress_keys(const uint16_t *k_bits, int32_t Hkv, int32_t l, int32_t d,
                             int32_t p, int32_t s, double *ck_f64, uint16_t *ck_bits) {
    int32_t n_c = oracle_num_kernels(l, p, s);
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t jh = 0; jh < n_c; ++jh)
            for (int32_t c = 0; c < d; ++c) {
                double sum = 0.0;
                for (int32_t t = jh * s; t < jh * s + p; ++t)
                    sum += bf16_to_f64(k_bits[((size_t)h * l + t) * d + c]);
                double mean = sum / (double)p;
                size_t o = ((size_t)h * n_c + jh) * d + c;
                if (ck_f64) ck_f64[o] = mean;
                if (ck_bits) ck_bits[o] = f64_to_bf16(mean);
            }
    return n_c;
}

/* ---- coarse semantic kernels for the approximate log-sum-exp ------------------ */

/* Number of coarse kernels whose rho fine kernels rho*c, rho*c+2, .., rho*c+2(rho-1) all lie
 * among the first n fine kernels ("Efficient Top-K Implementation": coarse-grained semantic
 * kernels of size s_c >> s). */
int32_t oracle_num_coarse(int32_t n, int32_t rho) {
    if (rho < 1 || n < 2 * rho - 1) return 0;
    return (n - (2 * rho - 1)) / rho + 1;
}

/* CKc[h, c, :] = mean_r CK[h, rho*c + 2r, :], r = 0..rho-1, from the bf16 fine representations.
 *   ck_bits   [Hkv, n_c, d]
 *   ckc_f64   [Hkv, n_cc, d] unrounded (may be NULL); ckc_bits rounded to bf16 (may be NULL)
 * Returns n_cc = oracle_num_coarse(n_c, rho). */
int32_t oracle_coarse_kernels(const uint16_t *ck_bits, int32_t Hkv, int32_t n_c, int32_t d,
                              int32_t rho, double *ckc_f64, uint16_t *ckc_bits) {
    int32_t n_cc = oracle_num_coarse(n_c, rho);
    for (int32_t h = 0; h < Hkv; ++h)
        for (int32_t c = 0; c < n_cc; ++c)
            for (int32_t e = 0; e < d; ++e) {
                double sum = 0.0;
                for (int32_t r = 0; r < rho; ++r)
                    sum += bf16_to_f64(ck_bits[((size_t)h * n_c + (size_t)rho * c + 2 * r) * d + e]);
                double mean = sum / (double)rho;
                size_t o = ((size_t)h * n_cc + c) * d + e;
                if (ckc_f64) ckc_f64[o] = mean;
                if (ckc_bits) ckc_bits[o] = f64_to_bf16(mean);
            }
    return n_cc;
}

/* ---- O2: kernel relevance for one query row ------------------------------- */

/* r[jh] = (1/G) sum_g softmax_jh(scale * <q_g, CK[jh]>), jh < n_vis, then floored.
 * (section 2.1.2: r_kernel; "Top-K Blocks Sharing": mean over the group;
 * "Efficient Top-K Implementation": softmax first, then aggregate.)
 *   q_row   G consecutive heads of one token, [G, d] bf16 bits
 *   ck_h    [n_c, d] bf16 bits of this key-value head
 *   r       [n_vis] out
 *   z, e    scratch of n_vis doubles each */
static void kernel_scores_row(const uint16_t *q_row, const uint16_t *ck_h, int32_t G, int32_t d,
                              int32_t n_vis, double scale, double *r, double *z) {
    for (int32_t jh = 0; jh < n_vis; ++jh) r[jh] = 0.0;
    for (int32_t g = 0; g < G; ++g) {
        double zmax = -INFINITY;
        for (int32_t jh = 0; jh < n_vis; ++jh) {
            double dot = 0.0;
            for (int32_t c = 0; c < d; ++c)
                dot += bf16_to_f64(q_row[(size_t)g * d + c]) * bf16_to_f64(ck_h[(size_t)jh * d + c]);
            z[jh] = scale * dot;
            if (z[jh] > zmax) zmax = z[jh];
        }
        double denom = 0.0;
        for (int32_t jh = 0; jh < n_vis; ++jh) denom += exp(z[jh] - zmax);
        for (int32_t jh = 0; jh < n_vis; ++jh) r[jh] += exp(z[jh] - zmax) / denom;
    }
    for (int32_t jh = 0; jh < n_vis; ++jh) {
        r[jh] /= (double)G;
        if (r[jh] < ORACLE_SCORE_FLOOR) r[jh] = ORACLE_SCORE_FLOOR;
    }
}

/* The same with the approximate log-sum-exp: per head, lse = log sum over the n_vis_c visible
 * coarse kernels of exp(scale <q_g, CKc>) + log(rho) (0 when none is visible), and
 * r[jh] = (1/G) sum_g exp(scale <q_g, CK[jh]> - lse_g), clamped to [2^-100, 2^100].
 *   ckc_h   [n_cc, d] bf16 bits of the coarse kernels of this key-value head
 *   lse_out [G] (may be NULL): the approximate log-sum-exp per head */
static void kernel_scores_row_coarse(const uint16_t *q_row, const uint16_t *ck_h, const uint16_t *ckc_h,
                                     int32_t G, int32_t d, int32_t n_vis, int32_t n_vis_c, int32_t rho,
                                     double scale, double *r, double *z, double *lse_out) {
    for (int32_t jh = 0; jh < n_vis; ++jh) r[jh] = 0.0;
    for (int32_t g = 0; g < G; ++g) {
        double lse = 0.0;
        if (n_vis_c > 0) {
            double zmax = -INFINITY;
            for (int32_t c = 0; c < n_vis_c; ++c) {
                double dot = 0.0;
                for (int32_t e = 0; e < d; ++e)
                    dot += bf16_to_f64(q_row[(size_t)g * d + e]) * bf16_to_f64(ckc_h[(size_t)c * d + e]);
                z[c] = scale * dot;
                if (z[c] > zmax) zmax = z[c];
            }
            double denom = 0.0;
            for (int32_t c = 0; c < n_vis_c; ++c) denom += exp(z[c] - zmax);
            lse = zmax + log(denom) + log((double)rho);
        }
        if (lse_out) lse_out[g] = lse;
        for (int32_t jh = 0; jh < n_vis; ++jh) {
            double dot = 0.0;
            for (int32_t e = 0; e < d; ++e)
                dot += bf16_to_f64(q_row[(size_t)g * d + e]) * bf16_to_f64(ck_h[(size_t)jh * d + e]);
            r[jh] += exp(scale * dot - lse);
        }
    }
    for (int32_t jh = 0; jh < n_vis; ++jh) {
        r[jh] /= (double)G;
        if (r[jh] < ORACLE_SCORE_FLOOR) r[jh] = ORACLE_SCORE_FLOOR;
        if (r[jh] > ORACLE_SCORE_CEIL) r[jh] = ORACLE_SCORE_CEIL;
    }
}

/* Group-mean kernel scores for a list of query rows (for tests and small cases).
 *   q_bits    [Tq, Hq, d]; row t is the query at position pos[t]
 *   ck_bits   [Hkv, n_c, d]
 *   r_out     [Hkv, Tq, n_c] fp64; entries jh >= n_vis(pos[t]) are set to 0 */
void oracle_kernel_scores(const uint16_t *q_bits, const uint16_t *ck_bits, const int32_t *pos,
                          int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c,
                          int32_t p, int32_t s, double scale, double *r_out) {
    int32_t G = Hq / Hkv;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(n_c > 0 ? n_c : 1));
#pragma omp for schedule(dynamic, 16)
        for (int32_t t = 0; t < Tq; ++t)
            for (int32_t h = 0; h < Hkv; ++h) {
                int32_t n_vis = oracle_num_kernels(pos[t] + 1, p, s);
                if (n_vis > n_c) n_vis = n_c;
                double *r = r_out + ((size_t)h * Tq + t) * n_c;
                for (int32_t jh = 0; jh < n_c; ++jh) r[jh] = 0.0;
                kernel_scores_row(q_bits + ((size_t)t * Hq + (size_t)h * G) * d,
                                  ck_bits + (size_t)h * n_c * d, G, d, n_vis, scale, r, z);
            }
        free(z);
    }
}

/* Group-mean kernel scores with the approximate log-sum-exp, for a list of query rows.
 *   ckc_bits  [Hkv, n_cc, d] coarse kernels (oracle_coarse_kernels)
 *   r_out     [Hkv, Tq, n_c]; lse_out [Hkv, Tq, G] (may be NULL) */
void oracle_kernel_scores_coarse(const uint16_t *q_bits, const uint16_t *ck_bits, const uint16_t *ckc_bits,
                                 const int32_t *pos, int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d,
                                 int32_t n_c, int32_t n_cc, int32_t p, int32_t s, int32_t rho, double scale,
                                 double *r_out, double *lse_out) {
    int32_t G = Hq / Hkv;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(n_c > 0 ? n_c : 1));
#pragma omp for schedule(dynamic, 16)
        for (int32_t t = 0; t < Tq; ++t)
            for (int32_t h = 0; h < Hkv; ++h) {
                int32_t n_vis = oracle_num_kernels(pos[t] + 1, p, s);
                if (n_vis > n_c) n_vis = n_c;
                int32_t n_vis_c = oracle_num_coarse(n_vis, rho);
                double *r = r_out + ((size_t)h * Tq + t) * n_c;
                for (int32_t jh = 0; jh < n_c; ++jh) r[jh] = 0.0;
                kernel_scores_row_coarse(q_bits + ((size_t)t * Hq + (size_t)h * G) * d,
                                         ck_bits + (size_t)h * n_c * d, ckc_bits + (size_t)h * n_cc * d, G, d,
                                         n_vis, n_vis_c, rho, scale, r, z,
                                         lse_out ? lse_out + ((size_t)h * Tq + t) * G : NULL);
            }
        free(z);
    }
}

/* ---- O3: block relevance and selection ------------------------------------ */

/* Eq. (1): R[j] = max over visible kernels jh whose token span [jh*s, jh*s+p)
 * intersects the block's span [j*m, (j+1)*m); -inf when no visible kernel does.
 * The test is the literal interval intersection, not a closed-form window. */
static void block_scores_row(const double *r, int32_t n_vis, int32_t n_blk, int32_t m, int32_t p,
                             int32_t s, double *R) {
    for (int32_t j = 0; j < n_blk; ++j) {
        double best = -INFINITY;
        int64_t b_lo = (int64_t)j * m, b_hi = (int64_t)(j + 1) * m;      /* [b_lo, b_hi) */
        for (int32_t jh = 0; jh < n_vis; ++jh) {
            int64_t k_lo = (int64_t)jh * s, k_hi = k_lo + p;             /* [k_lo, k_hi) */
            int intersects = (k_lo < b_hi) && (b_lo < k_hi);
            if (intersects && r[jh] > best) best = r[jh];
        }
        R[j] = best;
    }
}

/* Select blocks for a list of query rows of one sequence.
 *   q_bits     [Tq, Hq, d]; row t is the query at position pos[t]
 *   ck_bits    [Hkv, n_c, d] compressed keys (bf16) of the sequence
 *   block_idx  [Hkv, Tq, topk] out: selected block indices ascending, -1 padded
 *   margins    [Hkv, Tq, 2] out (may be NULL): smallest selected non-forced score and
 *              largest unselected score (NaN when there is none)
 *   R_out      [Hkv, Tq, nb_cap] out (may be NULL): block scores after forcing
 *              (+inf forced, -inf no visible kernel, NaN beyond the query's own block)
 * Section 2.1.2: "selects the k blocks with the highest relevance"; the initial and the
 * local-window blocks get score infinity; with at most k blocks everything is selected. */
static void select_rows(const uint16_t *q_bits, const uint16_t *ck_bits, const int32_t *pos,
                        int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c,
                        int32_t m, int32_t p, int32_t s, int32_t topk, int32_t n_init,
                        int32_t n_local, double scale, int32_t *block_idx, double *margins,
                        double *R_out, int32_t nb_cap, int32_t rho, const uint16_t *ckc_bits, int32_t n_cc) {
    int32_t G = Hq / Hkv;
#pragma omp parallel
    {
        int32_t max_blk = 1;
        for (int32_t t = 0; t < Tq; ++t)
            if (pos[t] / m + 1 > max_blk) max_blk = pos[t] / m + 1;
        double *z = (double *)malloc(sizeof(double) * (size_t)(n_c > 0 ? n_c : 1));
        double *r = (double *)malloc(sizeof(double) * (size_t)(n_c > 0 ? n_c : 1));
        double *R = (double *)malloc(sizeof(double) * (size_t)max_blk);
        char *taken = (char *)malloc((size_t)max_blk);
#pragma omp for schedule(dynamic, 4)
        for (int32_t t = 0; t < Tq; ++t)
            for (int32_t h = 0; h < Hkv; ++h) {
                int32_t i = pos[t];
                int32_t b_i = i / m;               /* the query's own block          */
                int32_t n_blk = b_i + 1;           /* candidate blocks 0..b_i        */
                int32_t n_vis = oracle_num_kernels(i + 1, p, s);
                if (n_vis > n_c) n_vis = n_c;
                if (ckc_bits)      /* approximate log-sum-exp from the coarse kernels */
                    kernel_scores_row_coarse(q_bits + ((size_t)t * Hq + (size_t)h * G) * d,
                                             ck_bits + (size_t)h * n_c * d, ckc_bits + (size_t)h * n_cc * d,
                                             G, d, n_vis, oracle_num_coarse(n_vis, rho), rho, scale, r, z, NULL);
                else
                    kernel_scores_row(q_bits + ((size_t)t * Hq + (size_t)h * G) * d,
                                      ck_bits + (size_t)h * n_c * d, G, d, n_vis, scale, r, z);
                block_scores_row(r, n_vis, n_blk, m, p, s, R);
                for (int32_t j = 0; j < n_blk; ++j) {
                    int forced = (j < n_init) || (j > b_i - n_local);
                    if (forced) R[j] = INFINITY;
                    taken[j] = 0;
                }
                int32_t n_sel = topk < n_blk ? topk : n_blk;
                double kth = NAN;                  /* smallest selected unforced score */
                for (int32_t c = 0; c < n_sel; ++c) {
                    int32_t best = -1;
                    for (int32_t j = 0; j < n_blk; ++j)   /* strict > : lower index wins ties */
                        if (!taken[j] && (best < 0 || R[j] > R[best])) best = j;
                    taken[best] = 1;
                    if (R[best] != INFINITY) kth = R[best];
                }
                double next = NAN;                 /* largest score left out         */
                for (int32_t j = 0; j < n_blk; ++j)
                    if (!taken[j] && (isnan(next) || R[j] > next)) next = R[j];
                int32_t *out = block_idx + ((size_t)h * Tq + t) * topk;
                int32_t w = 0;
                for (int32_t j = 0; j < n_blk; ++j)
                    if (taken[j]) out[w++] = j;
                for (; w < topk; ++w) out[w] = -1;
                if (margins) {
                    margins[((size_t)h * Tq + t) * 2 + 0] = kth;
                    margins[((size_t)h * Tq + t) * 2 + 1] = next;
                }
                if (R_out) {
                    double *Ro = R_out + ((size_t)h * Tq + t) * nb_cap;
                    for (int32_t j = 0; j < nb_cap; ++j) Ro[j] = j < n_blk ? R[j] : NAN;
                }
            }
        free(z); free(r); free(R); free(taken);
    }
}

void oracle_select_blocks(const uint16_t *q_bits, const uint16_t *ck_bits, const int32_t *pos,
                          int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t n_c,
                          int32_t m, int32_t p, int32_t s, int32_t topk, int32_t n_init,
                          int32_t n_local, double scale, int32_t *block_idx, double *margins,
                          double *R_out, int32_t nb_cap) {
    select_rows(q_bits, ck_bits, pos, Tq, Hq, Hkv, d, n_c, m, p, s, topk, n_init, n_local, scale, block_idx,
                margins, R_out, nb_cap, 1, NULL, 0);
}

/* The same selection with the approximate log-sum-exp ("Efficient Top-K Implementation"):
 * ckc_bits [Hkv, n_cc, d] are the coarse kernels of ratio rho (oracle_coarse_kernels). */
void oracle_select_blocks_coarse(const uint16_t *q_bits, const uint16_t *ck_bits, const uint16_t *ckc_bits,
                                 const int32_t *pos, int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d,
                                 int32_t n_c, int32_t n_cc, int32_t m, int32_t p, int32_t s, int32_t topk,
                                 int32_t n_init, int32_t n_local, int32_t rho, double scale,
                                 int32_t *block_idx, double *margins, double *R_out, int32_t nb_cap) {
    select_rows(q_bits, ck_bits, pos, Tq, Hq, Hkv, d, n_c, m, p, s, topk, n_init, n_local, scale, block_idx,
                margins, R_out, nb_cap, rho, ckc_bits, n_cc);
}

/* ---- O4: attention over the selected blocks -------------------------------- */

/* o_i = sum_{t in T_i} softmax_t(scale * <q_i, k_t>) v_t,  T_i = { t <= i : floor(t/m) in Sel(i) },
 * LSE_i = log sum_{t in T_i} exp(scale * <q_i, k_t>)      (section 2.1.1, second stage).
 *   q_bits     [Tq, Hq, d]; row t is the query at position pos[t]
 *   k_bits, v_bits [Hkv, l, d]
 *   block_idx  [Hkv, Tq, topk], -1 entries ignored
 *   out        [Tq, Hq, d] fp64,  lse [Tq, Hq] fp64 (natural log)
 *   probs_sum  [Tq, Hq] fp64 (may be NULL): sum of the softmax weights, for the row-sum pin */
static void attend_rows(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits,
                        const int32_t *pos, const int32_t *block_idx, int32_t Tq, int32_t Hq,
                        int32_t Hkv, int32_t d, int32_t l, int32_t m, int32_t topk, double scale,
                        double *out, double *lse, double *probs_sum, int32_t l_ctx,
                        const uint64_t *tree_mask) {
    int32_t G = Hq / Hkv;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)topk * m);
        int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)topk * m);
#pragma omp for schedule(dynamic, 4)
        for (int32_t t = 0; t < Tq; ++t)
            for (int32_t hq = 0; hq < Hq; ++hq) {
                int32_t h = hq / G;
                int32_t i = pos[t];
                const uint16_t *q = q_bits + ((size_t)t * Hq + hq) * d;
                const int32_t *sel = block_idx + ((size_t)h * Tq + t) * topk;
                int32_t n = 0;
                for (int32_t c = 0; c < topk; ++c) {
                    if (sel[c] < 0) continue;
                    for (int32_t u = sel[c] * m; u < (sel[c] + 1) * m; ++u) {
                        int allowed;
                        if (!tree_mask) allowed = u <= i;       /* causal */
                        else allowed = u < l_ctx ||             /* context, or a draft token the mask lets through */
                                       (u - l_ctx < 64 && ((tree_mask[t] >> (u - l_ctx)) & 1u));
                        if (allowed && u < l) tok[n++] = u;     /* inside the cache */
                    }
                }
                double zmax = -INFINITY;
                for (int32_t a = 0; a < n; ++a) {
                    const uint16_t *kr = k_bits + ((size_t)h * l + tok[a]) * d;
                    double dot = 0.0;
                    for (int32_t c = 0; c < d; ++c) dot += bf16_to_f64(q[c]) * bf16_to_f64(kr[c]);
                    z[a] = scale * dot;
                    if (z[a] > zmax) zmax = z[a];
                }
                double denom = 0.0;
                for (int32_t a = 0; a < n; ++a) denom += exp(z[a] - zmax);
                double *o = out + ((size_t)t * Hq + hq) * d;
                for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
                double wsum = 0.0;
                for (int32_t a = 0; a < n; ++a) {
                    double w = exp(z[a] - zmax) / denom;
                    wsum += w;
                    const uint16_t *vr = v_bits + ((size_t)h * l + tok[a]) * d;
                    for (int32_t c = 0; c < d; ++c) o[c] += w * bf16_to_f64(vr[c]);
                }
                lse[(size_t)t * Hq + hq] = n > 0 ? zmax + log(denom) : -INFINITY;
                if (probs_sum) probs_sum[(size_t)t * Hq + hq] = wsum;
            }
        free(z); free(tok);
    }
}

void oracle_sparse_attn(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits,
                        const int32_t *pos, const int32_t *block_idx, int32_t Tq, int32_t Hq,
                        int32_t Hkv, int32_t d, int32_t l, int32_t m, int32_t topk, double scale,
                        double *out, double *lse, double *probs_sum) {
    attend_rows(q_bits, k_bits, v_bits, pos, block_idx, Tq, Hq, Hkv, d, l, m, topk, scale, out, lse,
                probs_sum, 0, NULL);
}

/* Tree-style draft verification (section 4.1, "InfLLM v2 for Target Model"): the Tq = n <= 64
 * drafted tokens occupy cache positions l_ctx .. l_ctx+n-1, query t is draft token t, and inside
 * that last n x n region the causal triangle is replaced by a mask: query t attends draft token j
 * iff bit j of tree_mask[t] is set.  Context tokens (< l_ctx) of the selected blocks are always
 * attended.  Everything else (block selection per token by position, scale, LSE) is unchanged;
 * a lower-triangular mask gives back oracle_sparse_attn. */
void oracle_sparse_attn_tree(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits,
                             const int32_t *block_idx, const uint64_t *tree_mask, int32_t n, int32_t l_ctx,
                             int32_t Hq, int32_t Hkv, int32_t d, int32_t l, int32_t m, int32_t topk,
                             double scale, double *out, double *lse) {
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (int32_t t = 0; t < n; ++t) pos[t] = l_ctx + t;
    attend_rows(q_bits, k_bits, v_bits, pos, block_idx, n, Hq, Hkv, d, l, m, topk, scale, out, lse, NULL,
                l_ctx, tree_mask);
    free(pos);
}

/* ---- O5: backward of the sparse attention ------------------------------------------------ */

/* Gradients of oracle_sparse_attn's output with respect to q, k and v for a given upstream
 * gradient dout, the block sets held fixed (section 2.1: the sparse attention is trainable; the
 * selection is a discrete choice and the mean-pooled kernels have no parameters, so the
 * gradient reaches q, k, v through the attention only.  The report prints no backward formulas;
 * these are the derivatives of the forward definition):
 *     p[t]   = softmax over T_i of z[t],  z[t] = scale <q_i, k_t>
 *     dv_t  += p[t] dout_i                       dp[t] = <dout_i, v_t>
 *     ds[t]  = p[t] (dp[t] - sum_u p[u] dp[u])
 *     dq_i   = scale sum_t ds[t] k_t             dk_t += scale ds[t] q_i
 * summed over the query heads of a group for dk, dv.
 *   dout_bits [Tq, Hq, d] bf16;  dq [Tq, Hq, d], dk, dv [Hkv, l, d] fp64 out (overwritten).
 * Optional (all three or none, NULL to skip): the size of the terms behind every gradient
 * element, the scale a rounding-error tolerance has to be measured in.  An implementation that
 * takes D = <dout_i, out_i> from a rounded copy of the output perturbs every ds[t] by p[t] dD,
 * with |dD| <= eps * A_i,  A_i = sum_t p[t] <|dout_i|, |v_t|>:
 *     dq_mag_i = scale sum_t (|ds[t]| + p[t] A_i) |k_t|
 *     dk_mag_t = scale sum   (|ds[t]| + p[t] A_i) |q_i|
 *     dv_mag_t =       sum    p[t] |dout_i| */
void oracle_sparse_attn_bwd(const uint16_t *q_bits, const uint16_t *k_bits, const uint16_t *v_bits,
                            const uint16_t *dout_bits, const int32_t *pos, const int32_t *block_idx,
                            int32_t Tq, int32_t Hq, int32_t Hkv, int32_t d, int32_t l, int32_t m,
                            int32_t topk, double scale, double *dq, double *dk, double *dv,
                            double *dq_mag, double *dk_mag, double *dv_mag) {
    int32_t G = Hq / Hkv;
    size_t kv_elems = (size_t)Hkv * l * d;
    int want_mag = dq_mag && dk_mag && dv_mag;
    for (size_t x = 0; x < kv_elems; ++x) dk[x] = dv[x] = 0.0;
    if (want_mag)
        for (size_t x = 0; x < kv_elems; ++x) dk_mag[x] = dv_mag[x] = 0.0;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)topk * m);
        double *dp = (double *)malloc(sizeof(double) * (size_t)topk * m);
        double *dpa = (double *)malloc(sizeof(double) * (size_t)topk * m);
        int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)topk * m);
        double *dk_own = (double *)calloc(kv_elems, sizeof(double));   /* this thread's share of the sums */
        double *dv_own = (double *)calloc(kv_elems, sizeof(double));
        double *dkm_own = want_mag ? (double *)calloc(kv_elems, sizeof(double)) : NULL;
        double *dvm_own = want_mag ? (double *)calloc(kv_elems, sizeof(double)) : NULL;
#pragma omp for schedule(dynamic, 4)
        for (int32_t t = 0; t < Tq; ++t)
            for (int32_t hq = 0; hq < Hq; ++hq) {
                int32_t h = hq / G;
                int32_t i = pos[t];
                const uint16_t *q = q_bits + ((size_t)t * Hq + hq) * d;
                const uint16_t *go = dout_bits + ((size_t)t * Hq + hq) * d;
                const int32_t *sel = block_idx + ((size_t)h * Tq + t) * topk;
                int32_t n = 0;
                for (int32_t c = 0; c < topk; ++c) {
                    if (sel[c] < 0) continue;
                    for (int32_t u = sel[c] * m; u < (sel[c] + 1) * m; ++u)
                        if (u <= i && u < l) tok[n++] = u;
                }
                double zmax = -INFINITY, denom = 0.0, pdp = 0.0;
                for (int32_t a = 0; a < n; ++a) {
                    const uint16_t *kr = k_bits + ((size_t)h * l + tok[a]) * d;
                    const uint16_t *vr = v_bits + ((size_t)h * l + tok[a]) * d;
                    double dot = 0.0, gv = 0.0, gva = 0.0;
                    for (int32_t c = 0; c < d; ++c) {
                        dot += bf16_to_f64(q[c]) * bf16_to_f64(kr[c]);
                        gv += bf16_to_f64(go[c]) * bf16_to_f64(vr[c]);
                        gva += fabs(bf16_to_f64(go[c]) * bf16_to_f64(vr[c]));
                    }
                    p[a] = scale * dot;
                    dp[a] = gv;
                    dpa[a] = gva;
                    if (p[a] > zmax) zmax = p[a];
                }
                for (int32_t a = 0; a < n; ++a) denom += exp(p[a] - zmax);
                double A = 0.0;
                for (int32_t a = 0; a < n; ++a) {
                    p[a] = exp(p[a] - zmax) / denom;
                    pdp += p[a] * dp[a];
                    A += p[a] * dpa[a];
                }
                double *gq = dq + ((size_t)t * Hq + hq) * d;
                for (int32_t c = 0; c < d; ++c) gq[c] = 0.0;
                if (want_mag) {
                    double *gm = dq_mag + ((size_t)t * Hq + hq) * d;
                    for (int32_t c = 0; c < d; ++c) gm[c] = 0.0;
                    for (int32_t a = 0; a < n; ++a) {
                        double w = fabs(p[a] * (dp[a] - pdp)) + p[a] * A;
                        size_t row = ((size_t)h * l + tok[a]) * d;
                        for (int32_t c = 0; c < d; ++c) {
                            gm[c] += scale * w * fabs(bf16_to_f64(k_bits[row + c]));
                            dkm_own[row + c] += scale * w * fabs(bf16_to_f64(q[c]));
                            dvm_own[row + c] += p[a] * fabs(bf16_to_f64(go[c]));
                        }
                    }
                }
                for (int32_t a = 0; a < n; ++a) {
                    double ds = p[a] * (dp[a] - pdp);
                    size_t row = ((size_t)h * l + tok[a]) * d;
                    for (int32_t c = 0; c < d; ++c) {
                        gq[c] += scale * ds * bf16_to_f64(k_bits[row + c]);
                        dk_own[row + c] += scale * ds * bf16_to_f64(q[c]);
                        dv_own[row + c] += p[a] * bf16_to_f64(go[c]);
                    }
                }
            }
#pragma omp critical
        for (size_t x = 0; x < kv_elems; ++x) {
            dk[x] += dk_own[x];
            dv[x] += dv_own[x];
            if (want_mag) {
                dk_mag[x] += dkm_own[x];
                dv_mag[x] += dvm_own[x];
            }
        }
        free(p); free(dp); free(dpa); free(tok); free(dk_own); free(dv_own); free(dkm_own); free(dvm_own);
    }
}

/* Rounding helper exported for tests of the bf16 conversion itself. */
uint16_t oracle_f64_to_bf16(double x) { return f64_to_bf16(x); }
double oracle_bf16_to_f64(uint16_t b) { return bf16_to_f64(b); }
