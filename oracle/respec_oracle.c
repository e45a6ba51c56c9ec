/*
 * respec_oracle.c -- CPU oracle for the speculative-decoding verify step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct fp64 implementation of what the verify step computes, written from the
 * paper's statement of speculative decoding (Section 2.2: the draft/validate
 * procedure, the acceptance rule Eq. 1 and the residual distribution Eq. 2).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Parity pins (all functions here are pinned, none is "parity unpinned"):
 *   attention  -- dense numpy brute force on tiny shapes, closed forms (identical
 *                 keys => running mean of V, constant V, one visible key),
 *                 causality and GQA-sharing invariants, split/merge identity,
 *                 a library routine (scaled_dot_product_attention) for one query.
 *   sampler    -- q == p accepts every draft, k = 0 equals numpy's
 *                 cumsum/searchsorted sampler, chi-square of the emitted-token
 *                 marginal against p over 10^6 draws, acceptance rate against
 *                 1 - TV(p,q), disjoint supports, exact enumeration over a
 *                 stratified uniform grid.
 *   tree attention -- the chain mask reproduces the chain function bit for bit, dense
 *                 numpy with an explicit visibility matrix, invariance of a row to
 *                 nodes off its path.
 *   paged attention / commit -- dense numpy over a cache gathered by the test's own
 *                 indexing, invariance to a permutation of the physical pages and to
 *                 the page size, poisoned unused slots, a chain commit equals cutting
 *                 the length, a committed tree path attends like a cache built from
 *                 the accepted tokens only.
 *   KD rows     -- scipy's rel_entr, torch autograd of kl_div over log_softmax in fp64,
 *                 central differences of an independently written loss, q == p gives
 *                 zero loss and gradient, gradient rows sum to zero, a two-token closed form.
 *   greedy / per-sequence temperature -- numpy's argmax (first maximum) row by row,
 *                 the T -> 0 limit of the stochastic function on well separated logits,
 *                 a mixed batch against the one-temperature function sequence by sequence.
 *   tree sampler -- a chain-shaped tree reproduces the chain function exactly, a
 *                 hand-worked case (tests/golden/tree_hand_case.json), chi-square of
 *                 the emitted token against p with three sibling candidates, the
 *                 closed-form probability that every sibling is rejected.
 *
 * Conventions (the paper fixes Eq. 1 and Eq. 2 only; the rest are this build's
 * stated readings):
 *   - Sequence b has R_b = q_indptr[b+1]-q_indptr[b] = k_b+1 query/target rows and
 *     L_b = kv_indptr[b+1]-kv_indptr[b] cached tokens, the R_b new ones included.
 *     Query row i sits at absolute position L_b-R_b+i and sees keys 0..L_b-R_b+i.
 *   - Target row i is the distribution of the token that follows query row i, so
 *     it verifies drafted token i (i < k_b); row k_b is the bonus row.
 *   - Drafted tokens are tested in order; the first rejected one is replaced by
 *     one sample from the residual distribution and validation stops (Section 2.2,
 *     "Validation").  If none is rejected one bonus token is drawn from row k_b.
 *   - Randomness is supplied: accept iff u < min(1, p/q) (strict), and the single
 *     final draw per sequence is an inverse-CDF walk in ascending token id that
 *     returns the first x whose running sum exceeds u*Z (strict).
 *   - Temperature divides both target and drafter logits before the softmax.
 *   - flags bit0: an acceptance test had |u - min(1,rho)| <= 1e-6;
 *     flags bit1: u*Z lay within 1e-6*Z of an edge of the chosen token's CDF cell.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1
#define ORACLE_ERR_ALLOC 2
#define ORACLE_ERR_DATA 3

#define BOUNDARY_EPS 1e-6

static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int pick_threads(int n_threads)
{
#ifdef _OPENMP
    if (n_threads <= 0)
        n_threads = omp_get_max_threads();
    return n_threads;
#else
    (void)n_threads;
    return 1;
#endif
}

int respec_oracle_max_threads(void)
{
    return pick_threads(0);
}

/* ------------------------------------------------------------------------- */
/* Verify attention: the plain definition.                                    */
/*   o[i,h,:] = sum_j softmax_j(sm_scale * <q[i,h,:], k[j,h/G,:]>) v[j,h/G,:]  */
/*   over the keys j = 0 .. L_b - R_b + i of the row's own sequence.           */
/* Layouts: q, out [total_q, Hq, D]; k_cache, v_cache [total_kv, Hkv, D];      */
/* out in fp64; lse [total_q, Hq] fp64 or NULL (natural log of the softmax     */
/* denominator, in units of the scaled scores).                                */
/* ------------------------------------------------------------------------- */
/* With a tree of drafts (tree_mask != NULL) row i sees every key before the new tokens and,    */
/* among the R_b new tokens, exactly those whose bit is set in tree_mask[q0+i] (its ancestors  */
/* and itself); the chain is the mask with bits 0..i.                                          */
static int attention_one_sequence(const void *q, const void *k_cache, const void *v_cache,
                                  int32_t q0, int32_t R, int64_t kv0, int64_t L, double *out,
                                  double *lse, int32_t Hq, int32_t Hkv, int32_t D,
                                  double sm_scale, int dtype, const uint64_t *tree_mask)
{
    const int32_t G = Hq / Hkv;
    double *score = (double *)malloc((size_t)L * sizeof(double));
    if (!score)
        return ORACLE_ERR_ALLOC;
    for (int32_t i = 0; i < R; ++i) {
        const int64_t last_key = tree_mask ? L - 1 : L - R + i; /* inclusive */
        const int64_t first_new = L - R;
        for (int32_t h = 0; h < Hq; ++h) {
            const int32_t hk = h / G;
            const int64_t qoff = ((int64_t)(q0 + i) * Hq + h) * D;
            double m = -INFINITY;
            for (int64_t j = 0; j <= last_key; ++j) {
                if (tree_mask && j >= first_new && !((tree_mask[q0 + i] >> (j - first_new)) & 1u)) {
                    score[j] = -INFINITY; /* hidden from this row */
                    continue;
                }
                const int64_t koff = ((kv0 + j) * Hkv + hk) * D;
                double dot = 0.0;
                for (int32_t d = 0; d < D; ++d)
                    dot += load_elem(q, qoff + d, dtype) * load_elem(k_cache, koff + d, dtype);
                score[j] = sm_scale * dot;
                if (score[j] > m)
                    m = score[j];
            }
            double denom = 0.0;
            for (int64_t j = 0; j <= last_key; ++j) {
                score[j] = score[j] == -INFINITY ? 0.0 : exp(score[j] - m);
                denom += score[j];
            }
            double *o = out + qoff;
            for (int32_t d = 0; d < D; ++d)
                o[d] = 0.0;
            for (int64_t j = 0; j <= last_key; ++j) {
                if (score[j] == 0.0)
                    continue;
                const int64_t voff = ((kv0 + j) * Hkv + hk) * D;
                const double a = score[j] / denom;
                for (int32_t d = 0; d < D; ++d)
                    o[d] += a * load_elem(v_cache, voff + d, dtype);
            }
            if (lse)
                lse[(int64_t)(q0 + i) * Hq + h] = m + log(denom);
        }
    }
    free(score);
    return ORACLE_OK;
}

static int verify_attention_any(const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *q_indptr, const int64_t *kv_indptr, double *out,
                                double *lse, int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                                double sm_scale, int dtype, int n_threads, const uint64_t *tree_mask)
{
    if (!q || !k_cache || !v_cache || !q_indptr || !kv_indptr || !out)
        return ORACLE_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0)
        return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return ORACLE_ERR_ARG;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t R = q_indptr[b + 1] - q_indptr[b];
        const int64_t L = kv_indptr[b + 1] - kv_indptr[b];
        if (R < 1 || L < R || (tree_mask && R > 64))
            return ORACLE_ERR_DATA;
    }
    int status = ORACLE_OK;
    const int nt = pick_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
    for (int32_t b = 0; b < B; ++b) {
        const int rc = attention_one_sequence(q, k_cache, v_cache, q_indptr[b],
                                              q_indptr[b + 1] - q_indptr[b], kv_indptr[b],
                                              kv_indptr[b + 1] - kv_indptr[b], out, lse, Hq, Hkv,
                                              D, sm_scale, dtype, tree_mask);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

int respec_oracle_verify_attention(const void *q, const void *k_cache, const void *v_cache,
                                   const int32_t *q_indptr, const int64_t *kv_indptr, double *out,
                                   double *lse, int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                                   double sm_scale, int dtype, int n_threads)
{
    return verify_attention_any(q, k_cache, v_cache, q_indptr, kv_indptr, out, lse, B, Hq, Hkv, D,
                                sm_scale, dtype, n_threads, NULL);
}

/* Verify attention over a tree of drafts (Section 4.1: candidate branches validated in
 * parallel); tree_mask [total_q] as described above, at most 64 rows per sequence. */
int respec_oracle_verify_attention_tree(const void *q, const void *k_cache, const void *v_cache,
                                        const int32_t *q_indptr, const int64_t *kv_indptr,
                                        const uint64_t *tree_mask, double *out, double *lse,
                                        int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                                        double sm_scale, int dtype, int n_threads)
{
    if (!tree_mask)
        return ORACLE_ERR_ARG;
    return verify_attention_any(q, k_cache, v_cache, q_indptr, kv_indptr, out, lse, B, Hq, Hkv, D,
                                sm_scale, dtype, n_threads, tree_mask);
}

/* ------------------------------------------------------------------------- */
/* Paged KV cache (the cache the serving side manages, Sections 5.1 and 5.2;   */
/* the paper fixes no layout).  K and V live in pages of page_size tokens,     */
/* [num_pages, page_size, Hkv, D]; sequence b owns the page ids                */
/* page_table[page_indptr[b] .. page_indptr[b+1]) in token order and holds     */
/* kv_len[b] tokens (the R_b new ones included).  Attention over it is the     */
/* plain definition applied to the sequence's tokens gathered in order.        */
/* ------------------------------------------------------------------------- */
static size_t elem_bytes(int dtype) { return dtype == ORACLE_F32 ? 4u : 2u; }

int respec_oracle_verify_attention_paged(const void *q, const void *k_pages, const void *v_pages,
                                         const int32_t *q_indptr, const int32_t *page_indptr,
                                         const int32_t *page_table, const int32_t *kv_len,
                                         const uint64_t *tree_mask, double *out, double *lse,
                                         int32_t B, int32_t num_pages, int32_t page_size,
                                         int32_t Hq, int32_t Hkv, int32_t D, double sm_scale,
                                         int dtype, int n_threads)
{
    if (!q || !k_pages || !v_pages || !q_indptr || !page_indptr || !page_table || !kv_len || !out)
        return ORACLE_ERR_ARG;
    if (B <= 0 || num_pages <= 0 || page_size <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0)
        return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return ORACLE_ERR_ARG;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t R = q_indptr[b + 1] - q_indptr[b];
        const int64_t pages = page_indptr[b + 1] - page_indptr[b];
        if (R < 1 || kv_len[b] < R || (int64_t)kv_len[b] > pages * page_size || (tree_mask && R > 64))
            return ORACLE_ERR_DATA;
        for (int64_t i = 0; i * page_size < kv_len[b]; ++i) {
            const int32_t pg = page_table[page_indptr[b] + i];
            if (pg < 0 || pg >= num_pages)
                return ORACLE_ERR_DATA;
        }
    }
    int status = ORACLE_OK;
    const size_t tok_bytes = (size_t)Hkv * D * elem_bytes(dtype);
    const int nt = pick_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
    for (int32_t b = 0; b < B; ++b) {
        const int64_t L = kv_len[b];
        char *kseq = (char *)malloc((size_t)L * tok_bytes);
        char *vseq = (char *)malloc((size_t)L * tok_bytes);
        int rc = ORACLE_OK;
        if (!kseq || !vseq) {
            rc = ORACLE_ERR_ALLOC;
        } else {
            for (int64_t j = 0; j < L; ++j) { /* token j lives in slot j % page_size of page j / page_size */
                const int64_t pg = page_table[page_indptr[b] + j / page_size];
                const size_t src = ((size_t)pg * page_size + (size_t)(j % page_size)) * tok_bytes;
                memcpy(kseq + (size_t)j * tok_bytes, (const char *)k_pages + src, tok_bytes);
                memcpy(vseq + (size_t)j * tok_bytes, (const char *)v_pages + src, tok_bytes);
            }
            rc = attention_one_sequence(q, kseq, vseq, q_indptr[b], q_indptr[b + 1] - q_indptr[b], 0, L,
                                        out, lse, Hq, Hkv, D, sm_scale, dtype, tree_mask);
        }
        free(kseq);
        free(vseq);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* After validation (Section 2.2) the accepted drafts become part of the sequence and the rest
 * of the speculative tokens are dropped.  The new tokens of sequence b sit at positions
 * first_new + r (r = their row, first_new = kv_len[b] - R_b; row 0 is the last committed
 * token).  The accepted nodes are rows path[0] < path[1] < ... (a chain: 1, 2, ..., n_b; pass
 * path == NULL): the K/V of row path[j] moves to position first_new + 1 + j, and the length
 * becomes first_new + 1 + n_b.  The token drawn last has no K/V yet.  k_pages and v_pages are
 * changed in place; positions at or beyond the new length keep whatever they held. */
int respec_oracle_commit_accepted_paged(void *k_pages, void *v_pages, const int32_t *q_indptr,
                                        const int32_t *page_indptr, const int32_t *page_table,
                                        int32_t *kv_len, const int32_t *path, int32_t path_stride,
                                        const int32_t *num_accepted, int32_t B, int32_t num_pages,
                                        int32_t page_size, int32_t Hkv, int32_t D, int dtype)
{
    if (!k_pages || !v_pages || !q_indptr || !page_indptr || !page_table || !kv_len || !num_accepted)
        return ORACLE_ERR_ARG;
    if (B <= 0 || num_pages <= 0 || page_size <= 0 || Hkv <= 0 || D <= 0 || (path && path_stride < 1))
        return ORACLE_ERR_ARG;
    const size_t tok_bytes = (size_t)Hkv * D * elem_bytes(dtype);
    for (int32_t b = 0; b < B; ++b) {
        const int32_t R = q_indptr[b + 1] - q_indptr[b];
        const int32_t n = num_accepted[b];
        const int64_t first_new = (int64_t)kv_len[b] - R;
        if (R < 1 || first_new < 0 || n < 0 || n > R - 1 || (path && n > path_stride))
            return ORACLE_ERR_DATA;
        for (int32_t j = 0; j < n; ++j) {
            const int32_t r = path ? path[(int64_t)b * path_stride + j] : j + 1;
            if (r < j + 1 || r >= R || (j > 0 && path && r <= path[(int64_t)b * path_stride + j - 1]))
                return ORACLE_ERR_DATA;
            const int64_t from = first_new + r, to = first_new + 1 + j;
            if (from == to)
                continue;
            const int64_t pf = page_table[page_indptr[b] + from / page_size];
            const int64_t pt = page_table[page_indptr[b] + to / page_size];
            if (pf < 0 || pf >= num_pages || pt < 0 || pt >= num_pages)
                return ORACLE_ERR_DATA;
            const size_t src = ((size_t)pf * page_size + (size_t)(from % page_size)) * tok_bytes;
            const size_t dst = ((size_t)pt * page_size + (size_t)(to % page_size)) * tok_bytes;
            memmove((char *)k_pages + dst, (const char *)k_pages + src, tok_bytes);
            memmove((char *)v_pages + dst, (const char *)v_pages + src, tok_bytes);
        }
        kv_len[b] = (int32_t)(first_new + 1 + n);
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Rejection sampling (Section 2.2, Eq. 1 and Eq. 2), one sequence at a time. */
/* ------------------------------------------------------------------------- */

/* p[x] = softmax(logits[row, :] / T)[x], max-subtracted, all in fp64. */
static void softmax_row(const void *logits, int64_t row, int64_t ld, int32_t V, double T,
                        int dtype, double *p)
{
    double m = -INFINITY;
    for (int32_t x = 0; x < V; ++x) {
        p[x] = load_elem(logits, row * ld + x, dtype) / T;
        if (p[x] > m)
            m = p[x];
    }
    double s = 0.0;
    for (int32_t x = 0; x < V; ++x) {
        p[x] = exp(p[x] - m);
        s += p[x];
    }
    for (int32_t x = 0; x < V; ++x)
        p[x] /= s;
}

/* First token whose running sum of w, in ascending id, exceeds u*Z. */
static int32_t inverse_cdf(const double *w, int32_t V, double Z, double u, int *near_edge)
{
    const double t = u * Z;
    double c = 0.0;
    int32_t last_positive = -1;
    for (int32_t x = 0; x < V; ++x) {
        const double before = c;
        c += w[x];
        if (w[x] > 0.0)
            last_positive = x;
        if (c > t) {
            const double lo = fabs(t - before), hi = fabs(c - t);
            if ((lo < hi ? lo : hi) <= BOUNDARY_EPS * Z)
                *near_edge = 1;
            return x;
        }
    }
    /* u*Z rounded up to the total: only reachable through rounding, always flagged */
    *near_edge = 1;
    return last_positive >= 0 ? last_positive : V - 1;
}

static int sample_one_sequence(const void *target_logits, const void *draft_logits,
                               const int32_t *draft_tokens, int32_t row0, int32_t drow0,
                               int32_t k, const float *u_accept, float u_final,
                               int32_t *out_tokens /* [max_k+1] */, int32_t *out_num_accepted,
                               int32_t *out_flags, int32_t max_k, int32_t V, int64_t ld_t,
                               int64_t ld_d, double T, int dtype)
{
    double *p = (double *)malloc((size_t)V * sizeof(double));
    double *q = (double *)malloc((size_t)V * sizeof(double));
    if (!p || !q) {
        free(p);
        free(q);
        return ORACLE_ERR_ALLOC;
    }
    int flag_accept = 0, flag_cdf = 0;
    int32_t n = 0, final_token = -1;
    int rejected = 0;
    for (int32_t j = 0; j <= max_k; ++j)
        out_tokens[j] = -1;

    for (int32_t i = 0; i < k; ++i) {
        softmax_row(target_logits, row0 + i, ld_t, V, T, dtype, p);
        softmax_row(draft_logits, drow0 + i, ld_d, V, T, dtype, q);
        const int32_t x = draft_tokens[drow0 + i];
        if (x < 0 || x >= V) {
            free(p);
            free(q);
            return ORACLE_ERR_DATA;
        }
        double rho;
        if (q[x] == 0.0)
            rho = p[x] > 0.0 ? INFINITY : 0.0;
        else
            rho = p[x] / q[x];
        const double thr = rho < 1.0 ? rho : 1.0;
        const double u = (double)u_accept[drow0 + i];
        if (fabs(u - thr) <= BOUNDARY_EPS)
            flag_accept = 1;
        if (u < thr) { /* Eq. 1: accepted, go on to the next drafted token */
            out_tokens[i] = x;
            n = i + 1;
            continue;
        }
        /* first rejection: one sample from the residual, Eq. 2 */
        double Z = 0.0;
        for (int32_t y = 0; y < V; ++y) {
            const double w = p[y] - q[y];
            q[y] = w > 0.0 ? w : 0.0;
            Z += q[y];
        }
        if (!(Z > 0.0)) { /* cannot happen in exact arithmetic; fall back to p */
            memcpy(q, p, (size_t)V * sizeof(double));
            Z = 1.0;
        }
        final_token = inverse_cdf(q, V, Z, (double)u_final, &flag_cdf);
        rejected = 1;
        break;
    }
    if (!rejected) { /* all k accepted (or k == 0): bonus token from target row k */
        softmax_row(target_logits, row0 + k, ld_t, V, T, dtype, p);
        final_token = inverse_cdf(p, V, 1.0, (double)u_final, &flag_cdf);
    }
    out_tokens[n] = final_token;
    *out_num_accepted = n;
    if (out_flags)
        *out_flags = (flag_accept ? 1 : 0) | (flag_cdf ? 2 : 0);
    free(p);
    free(q);
    return ORACLE_OK;
}

/*
 * target_logits [total_q, V] (row stride ld_t), draft_logits [total_q-B, V] (ld_d);
 * draft rows of sequence b start at q_indptr[b]-b.  out_tokens [B, max_k+1].
 */
int respec_oracle_rejection_sample(const void *target_logits, const void *draft_logits,
                                   const int32_t *draft_tokens, const int32_t *q_indptr,
                                   const float *u_accept, const float *u_final,
                                   int32_t *out_tokens, int32_t *out_num_accepted,
                                   int32_t *out_flags, int32_t B, int32_t max_k, int32_t V,
                                   int64_t ld_t, int64_t ld_d, double temperature, int dtype,
                                   int n_threads)
{
    if (!target_logits || !q_indptr || !u_final || !out_tokens || !out_num_accepted)
        return ORACLE_ERR_ARG;
    if (B <= 0 || V <= 0 || max_k < 0 || ld_t < V || !(temperature > 0.0))
        return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return ORACLE_ERR_ARG;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t k = q_indptr[b + 1] - q_indptr[b] - 1;
        if (k < 0 || k > max_k)
            return ORACLE_ERR_DATA;
        if (k > 0 && (!draft_logits || !draft_tokens || !u_accept || ld_d < V))
            return ORACLE_ERR_ARG;
    }
    int status = ORACLE_OK;
    const int nt = pick_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
    for (int32_t b = 0; b < B; ++b) {
        const int32_t row0 = q_indptr[b];
        const int32_t k = q_indptr[b + 1] - row0 - 1;
        const int rc = sample_one_sequence(
            target_logits, draft_logits, draft_tokens, row0, row0 - b, k, u_accept, u_final[b],
            out_tokens + (int64_t)b * (max_k + 1), out_num_accepted + b,
            out_flags ? out_flags + b : NULL, max_k, V, ld_t, ld_d, temperature, dtype);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Greedy verification and one temperature per sequence.                       */
/* The paper runs its tasks at different sampling temperatures (Table 2) and   */
/* a rollout batch can mix them; temperature 0 means greedy decoding.  As T    */
/* goes to 0, softmax(z/T) tends to a point mass on the largest logit, so      */
/* Eq. 1 becomes "accept the drafted token iff it is the target's argmax" and  */
/* Eq. 2 becomes "replace it by the target's argmax"; the bonus token is the   */
/* argmax of row k_b.  Reading for ties (equal largest logits): the token with */
/* the lowest id counts as the argmax, and only that one is accepted.  No      */
/* uniform is read and no flag is raised for a greedy sequence.                */
/* ------------------------------------------------------------------------- */
static int32_t argmax_row(const void *logits, int64_t row, int64_t ld, int32_t V, int dtype)
{
    int32_t best = 0;
    double zbest = load_elem(logits, row * ld, dtype);
    for (int32_t x = 1; x < V; ++x) {
        const double z = load_elem(logits, row * ld + x, dtype);
        if (z > zbest) {
            zbest = z;
            best = x;
        }
    }
    return best;
}

static int greedy_one_sequence(const void *target_logits, const int32_t *draft_tokens, int32_t row0,
                               int32_t drow0, int32_t k, int32_t *out_tokens, int32_t *out_num_accepted,
                               int32_t *out_flags, int32_t max_k, int32_t V, int64_t ld_t, int dtype)
{
    for (int32_t j = 0; j <= max_k; ++j)
        out_tokens[j] = -1;
    int32_t n = 0;
    while (n < k) {
        const int32_t x = draft_tokens[drow0 + n];
        if (x < 0 || x >= V)
            return ORACLE_ERR_DATA;
        if (x != argmax_row(target_logits, row0 + n, ld_t, V, dtype))
            break;
        out_tokens[n] = x;
        ++n;
    }
    /* the replacement of the first rejected draft, or the bonus token: the argmax of row n */
    out_tokens[n] = argmax_row(target_logits, row0 + n, ld_t, V, dtype);
    *out_num_accepted = n;
    if (out_flags)
        *out_flags = 0;
    return ORACLE_OK;
}

/* As respec_oracle_rejection_sample, with temperature[b] per sequence; 0 selects greedy. */
int respec_oracle_rejection_sample_per_seq(const void *target_logits, const void *draft_logits,
                                           const int32_t *draft_tokens, const int32_t *q_indptr,
                                           const float *u_accept, const float *u_final,
                                           const float *temperature, int32_t *out_tokens,
                                           int32_t *out_num_accepted, int32_t *out_flags, int32_t B,
                                           int32_t max_k, int32_t V, int64_t ld_t, int64_t ld_d,
                                           int dtype, int n_threads)
{
    if (!target_logits || !q_indptr || !u_final || !temperature || !out_tokens || !out_num_accepted)
        return ORACLE_ERR_ARG;
    if (B <= 0 || V <= 0 || max_k < 0 || ld_t < V)
        return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return ORACLE_ERR_ARG;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t k = q_indptr[b + 1] - q_indptr[b] - 1;
        if (k < 0 || k > max_k)
            return ORACLE_ERR_DATA;
        if (!(temperature[b] >= 0.0f) || isinf(temperature[b]))
            return ORACLE_ERR_DATA;
        if (k > 0 && !draft_tokens)
            return ORACLE_ERR_ARG;
        if (k > 0 && temperature[b] > 0.0f && (!draft_logits || !u_accept || ld_d < V))
            return ORACLE_ERR_ARG;
    }
    int status = ORACLE_OK;
    const int nt = pick_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
    for (int32_t b = 0; b < B; ++b) {
        const int32_t row0 = q_indptr[b];
        const int32_t k = q_indptr[b + 1] - row0 - 1;
        int32_t *toks = out_tokens + (int64_t)b * (max_k + 1);
        int rc;
        if (temperature[b] == 0.0f)
            rc = greedy_one_sequence(target_logits, draft_tokens, row0, row0 - b, k, toks,
                                     out_num_accepted + b, out_flags ? out_flags + b : NULL, max_k, V,
                                     ld_t, dtype);
        else
            rc = sample_one_sequence(target_logits, draft_logits, draft_tokens, row0, row0 - b, k,
                                     u_accept, u_final[b], toks, out_num_accepted + b,
                                     out_flags ? out_flags + b : NULL, max_k, V, ld_t, ld_d,
                                     (double)temperature[b], dtype);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Rejection sampling over a tree of drafts.                                   */
/* The paper names the tree (branching factor t, Section 4.1) and refers to    */
/* its drafting method for the rest; this build's reading is the multi-round   */
/* form of Eq. 1 / Eq. 2 for sibling candidates drawn independently from the   */
/* same drafter distribution q:                                                */
/*   at a node, p_0 = p (target row of the node); its children are tried in    */
/*   ascending row order; child c with token x is accepted iff                 */
/*   u_c < min(1, p_r(x)/q(x)); a rejection replaces p_r by                    */
/*   p_{r+1} = max(0, p_r - q) / Z_{r+1}  (Eq. 2 applied again);               */
/*   an accepted child becomes the node (r back to 0); when no child is left   */
/*   one token is drawn from the current p_r and validation stops.             */
/* A chain (every node one child) is exactly the procedure above.              */
/* Rows of sequence b: q_indptr[b] .. , row 0 the root (last committed token), */
/* parent[row] the local index of the parent row (-1 for the root, < the row's */
/* own index otherwise).  target_logits, draft_logits [total_q, V]: row i is   */
/* the target / drafter distribution of the token that follows row i (drafter  */
/* rows of leaves are not read).  u_accept [total_q] (entry of the root        */
/* unused), u_final [B].  out_tokens [B, max_depth+1]; out_path [B, max_depth]  */
/* the local rows of the accepted nodes (-1 beyond).                           */
/* ------------------------------------------------------------------------- */
static int sample_one_tree(const void *target_logits, const void *draft_logits,
                           const int32_t *node_tokens, const int32_t *parent, int32_t row0,
                           int32_t R, const float *u_accept, float u_final, int32_t *out_tokens,
                           int32_t *out_path, int32_t *out_num_accepted, int32_t *out_flags,
                           int32_t max_depth, int32_t V, int64_t ld_t, int64_t ld_d, double T,
                           int dtype)
{
    double *p = (double *)malloc((size_t)V * sizeof(double));
    double *q = (double *)malloc((size_t)V * sizeof(double));
    if (!p || !q) {
        free(p);
        free(q);
        return ORACLE_ERR_ALLOC;
    }
    int flag_accept = 0, flag_cdf = 0;
    int32_t n = 0, cur = 0;
    for (int32_t j = 0; j <= max_depth; ++j)
        out_tokens[j] = -1;
    for (int32_t j = 0; j < max_depth; ++j)
        out_path[j] = -1;
    for (;;) {
        softmax_row(target_logits, row0 + cur, ld_t, V, T, dtype, p);
        int have_q = 0;
        int32_t next = -1;
        for (int32_t c = cur + 1; c < R && next < 0; ++c) {
            if (parent[row0 + c] != cur)
                continue;
            if (!have_q) {
                softmax_row(draft_logits, row0 + cur, ld_d, V, T, dtype, q);
                have_q = 1;
            }
            const int32_t x = node_tokens[row0 + c];
            if (x < 0 || x >= V || n >= max_depth) {
                free(p);
                free(q);
                return ORACLE_ERR_DATA;
            }
            double rho;
            if (q[x] == 0.0)
                rho = p[x] > 0.0 ? INFINITY : 0.0;
            else
                rho = p[x] / q[x];
            const double thr = rho < 1.0 ? rho : 1.0;
            const double u = (double)u_accept[row0 + c];
            if (fabs(u - thr) <= BOUNDARY_EPS)
                flag_accept = 1;
            if (u < thr) { /* accepted: the child becomes the node */
                out_tokens[n] = x;
                out_path[n] = c;
                n += 1;
                next = c;
                break;
            }
            /* rejected: p <- max(0, p - q) / Z  (Eq. 2 applied to the current p) */
            double Z = 0.0;
            for (int32_t y = 0; y < V; ++y) {
                const double w = p[y] - q[y];
                p[y] = w > 0.0 ? w : 0.0;
                Z += p[y];
            }
            if (!(Z > 0.0)) { /* cannot happen in exact arithmetic; keep the target itself */
                softmax_row(target_logits, row0 + cur, ld_t, V, T, dtype, p);
                flag_cdf = 1;
            } else {
                for (int32_t y = 0; y < V; ++y)
                    p[y] /= Z;
            }
        }
        if (next >= 0) {
            cur = next;
            continue;
        }
        /* no child left (or none offered): one draw from the current p */
        double Zp = 0.0;
        for (int32_t y = 0; y < V; ++y)
            Zp += p[y];
        out_tokens[n] = inverse_cdf(p, V, Zp, (double)u_final, &flag_cdf);
        break;
    }
    *out_num_accepted = n;
    if (out_flags)
        *out_flags = (flag_accept ? 1 : 0) | (flag_cdf ? 2 : 0);
    free(p);
    free(q);
    return ORACLE_OK;
}

int respec_oracle_tree_rejection_sample(const void *target_logits, const void *draft_logits,
                                        const int32_t *node_tokens, const int32_t *parent,
                                        const int32_t *q_indptr, const float *u_accept,
                                        const float *u_final, int32_t *out_tokens,
                                        int32_t *out_path, int32_t *out_num_accepted,
                                        int32_t *out_flags, int32_t B, int32_t max_depth,
                                        int32_t V, int64_t ld_t, int64_t ld_d,
                                        double temperature, int dtype, int n_threads)
{
    if (!target_logits || !draft_logits || !node_tokens || !parent || !q_indptr || !u_accept ||
        !u_final || !out_tokens || !out_path || !out_num_accepted)
        return ORACLE_ERR_ARG;
    if (B <= 0 || V <= 0 || max_depth < 0 || ld_t < V || ld_d < V || !(temperature > 0.0))
        return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return ORACLE_ERR_ARG;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t row0 = q_indptr[b], R = q_indptr[b + 1] - row0;
        if (R < 1 || parent[row0] != -1)
            return ORACLE_ERR_DATA;
        for (int32_t i = 1; i < R; ++i)
            if (parent[row0 + i] < 0 || parent[row0 + i] >= i)
                return ORACLE_ERR_DATA;
    }
    int status = ORACLE_OK;
    const int nt = pick_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
    for (int32_t b = 0; b < B; ++b) {
        const int32_t row0 = q_indptr[b];
        const int rc = sample_one_tree(
            target_logits, draft_logits, node_tokens, parent, row0, q_indptr[b + 1] - row0,
            u_accept, u_final[b], out_tokens + (int64_t)b * (max_depth + 1),
            out_path + (int64_t)b * (max_depth > 0 ? max_depth : 1), out_num_accepted + b,
            out_flags ? out_flags + b : NULL, max_depth, V, ld_t, ld_d, temperature, dtype);
        if (rc != ORACLE_OK) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Reward-weighted knowledge distillation of the drafter, one logits row at a  */
/* time (Section 5.3, "Reward-Weighted Knowledge Distillation"; Algorithm 1):  */
/*   loss_row = w * KL(p || q),  p = softmax(target row), q = softmax(draft    */
/*   row), and its gradient with respect to the drafter's logits, w * (q - p). */
/* w is the weight w(r) of the row's sample, supplied per row (the paper's     */
/* default w(r) = r with an unspecified normalisation and clipping is the      */
/* caller's).  Terms with p(x) = 0 contribute nothing.  total = sum of rows.   */
/* ------------------------------------------------------------------------- */
int respec_oracle_kd_rows(const void *target_logits, const void *draft_logits, const float *row_weight,
                          double *grad, double *row_loss, double *total_loss, int32_t rows, int32_t V,
                          int64_t ld_t, int64_t ld_d, int dtype, int n_threads)
{
    if (!target_logits || !draft_logits || !row_weight || !grad || !row_loss)
        return ORACLE_ERR_ARG;
    if (rows <= 0 || V <= 0 || ld_t < V || ld_d < V)
        return ORACLE_ERR_ARG;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return ORACLE_ERR_ARG;
    int status = ORACLE_OK;
    const int nt = pick_threads(n_threads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
    for (int32_t r = 0; r < rows; ++r) {
        double *p = (double *)malloc((size_t)V * sizeof(double));
        double *q = (double *)malloc((size_t)V * sizeof(double));
        if (!p || !q) {
#pragma omp critical
            status = ORACLE_ERR_ALLOC;
        } else {
            softmax_row(target_logits, r, ld_t, V, 1.0, dtype, p);
            softmax_row(draft_logits, r, ld_d, V, 1.0, dtype, q);
            const double w = (double)row_weight[r];
            double kl = 0.0;
            for (int32_t x = 0; x < V; ++x) {
                if (p[x] > 0.0)
                    kl += p[x] * (log(p[x]) - log(q[x]));
                grad[(int64_t)r * V + x] = w * (q[x] - p[x]);
            }
            row_loss[r] = w * kl;
        }
        free(p);
        free(q);
    }
    if (status == ORACLE_OK && total_loss) {
        double t = 0.0;
        for (int32_t r = 0; r < rows; ++r)
            t += row_loss[r];
        *total_loss = t;
    }
    return status;
}

/* softmax(logits[r,:]/T) for r in [0,n_rows), fp64 out [n_rows, V]; lets tests look inside. */
int respec_oracle_softmax_rows(const void *logits, int32_t n_rows, int32_t V, int64_t ld,
                               double temperature, int dtype, double *out)
{
    if (!logits || !out || n_rows < 0 || V <= 0 || ld < V || !(temperature > 0.0))
        return ORACLE_ERR_ARG;
    for (int32_t r = 0; r < n_rows; ++r)
        softmax_row(logits, r, ld, V, temperature, dtype, out + (int64_t)r * V);
    return ORACLE_OK;
}
