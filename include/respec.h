/*
 * respec.h -- C boundary of the MI355X (gfx950) speculative-decoding verify step.
 *
 * The verify step is the "Validation" half of the draft/validate cycle of Section 2.2:
 * the target model scores the k drafted tokens plus one in a single batched forward
 * (Figure 2), drafted tokens are accepted in order with probability min(1, p/q) (Eq. 1),
 * the first rejected one is replaced by a sample from the residual distribution
 * max(0, p-q)/sum (Eq. 2), and when nothing is rejected one more token is drawn from the
 * target.  This library holds the two data-parallel pieces of that step:
 *
 *   respec_verify_attention   the attention of that forward: (k_b+1) causal query rows per
 *                             sequence, grouped-query heads, ragged per-sequence KV cache;
 *   respec_rejection_sample   Eq. 1 / Eq. 2 over the vocabulary with supplied uniforms
 *                             (respec_rejection_sample_per_seq: one temperature per sequence, 0 = greedy);
 * their counterparts for a tree of drafts (Section 4.1), respec_verify_attention_tree and
 * respec_tree_rejection_sample, the paged-cache forms respec_verify_attention_paged and
 * respec_commit_accepted_paged, respec_kd_rows, the drafter's distillation loss over the
 * same logits rows (Section 5.3), and respec_solver_pick, the Solver's table look-up (host code).
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer (HIP global memory) unless it says "host".
 *     The caller owns all buffers; the library allocates and frees nothing on the device
 *     and keeps no state between calls (the profiling hook below aside).
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and never synchronise.  Inputs must stay valid and unchanged until
 *     the stream has passed the call.
 *   - The return value reports host-detectable errors only (bad scalars, null pointers,
 *     misaligned pointers, workspace too small, a failed launch).  On error nothing is
 *     launched.  respec_last_error() gives a thread-local text for the last failure.
 *   - Data errors the host cannot see (k_b+1 > L_b, a token id outside [0,V), NaN or +inf
 *     logits) are undefined behaviour as far as results go, but never read or write
 *     outside the buffers described by the arguments.
 *   - No C++ exceptions cross this boundary and nothing is printed.
 *
 * Notation: B sequences; sequence b has R_b = k_b+1 query/target rows
 * (R_b = q_indptr[b+1]-q_indptr[b]) and L_b cached tokens (kv_indptr), the R_b new tokens
 * included; total_q = sum R_b, total_kv = sum L_b; Hq query heads, Hkv KV heads,
 * G = Hq/Hkv, head size D, vocabulary V.
 */
#ifndef RESPEC_H
#define RESPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RESPEC_OK = 0,
    RESPEC_ERR_INVALID_ARG = 1, /* null/misaligned pointer, non-positive size, bad scalar */
    RESPEC_ERR_UNSUPPORTED = 2, /* valid request outside what the kernels cover         */
    RESPEC_ERR_WORKSPACE = 3,   /* workspace missing or smaller than *_workspace_bytes  */
    RESPEC_ERR_HIP = 4          /* the HIP runtime refused a launch                      */
} respec_status_t;

typedef enum { RESPEC_F32 = 0, RESPEC_BF16 = 1 } respec_dtype_t;

/* Static strings; never NULL. */
const char *respec_status_string(respec_status_t status);
/* Thread-local detail text of the calling thread's last failed call ("" if none). */
const char *respec_last_error(void);
/* major*10000 + minor*100 + patch */
int respec_version(void);

/*
 * Bytes of device workspace respec_verify_attention needs for any batch with these
 * host-side bounds (split-KV partial results).  All arguments are the same scalars the
 * call itself takes.  Returns 0 if the arguments are invalid or unsupported.
 */
size_t respec_verify_attention_workspace_bytes(int32_t B, int32_t total_q, int64_t total_kv,
                                               int32_t max_q_per_seq, int32_t max_kv_len,
                                               int32_t Hq, int32_t Hkv, int32_t D,
                                               respec_dtype_t dt);

/*
 * Verify attention (the attention inside the single target forward of Section 2.2 /
 * Figure 2; the paper fixes no layout, the ones below are this library's).
 *
 * For every sequence b, row i in [0,R_b) and query head h:
 *     out[q_indptr[b]+i, h, :] = sum_j softmax_j(sm_scale * <q[row,h,:], K_b[j,h/G,:]>) V_b[j,h/G,:]
 * over the keys j = 0 .. L_b-R_b+i of that sequence's cache (row i sits at absolute
 * position L_b-R_b+i; the cache already holds the K/V of the R_b new tokens; RoPE, if
 * any, is already applied).  Softmax and accumulation run in fp32; for RESPEC_BF16 the
 * products run on bf16 MFMA and the result is rounded to nearest-even bf16.
 *
 *   q         [total_q, Hq, D]    dt, contiguous, 16-byte aligned
 *   k_cache   [total_kv, Hkv, D]  dt, token-major, sequences back to back, 16-byte aligned
 *   v_cache   [total_kv, Hkv, D]  dt, same layout
 *   q_indptr  [B+1] int32, q_indptr[0] = 0, rows of sequence b = R_b >= 1
 *   kv_indptr [B+1] int64, kv_indptr[0] = 0, L_b >= R_b
 *   out       [total_q, Hq, D]    dt (written)
 *   lse       [total_q, Hq] f32 or NULL: natural log of the softmax denominator plus the
 *             row maximum, in units of the scaled scores (written when non-NULL)
 *   max_q_per_seq, max_kv_len   host-side upper bounds of R_b and L_b: they size the grid
 *             without a device synchronisation.  Rows or keys beyond them are NOT processed.
 *   D in {64, 128}; Hq % Hkv == 0; G * max_q_per_seq <= 256.
 *   workspace / workspace_bytes: at least respec_verify_attention_workspace_bytes(...)
 *             bytes, 256-byte aligned; contents are scratch.
 */
respec_status_t respec_verify_attention(const void *q, const void *k_cache, const void *v_cache,
                                        const int32_t *q_indptr, const int64_t *kv_indptr,
                                        void *out, float *lse, int32_t B, int32_t total_q,
                                        int64_t total_kv, int32_t max_q_per_seq,
                                        int32_t max_kv_len, int32_t Hq, int32_t Hkv, int32_t D,
                                        float sm_scale, respec_dtype_t dt, void *workspace,
                                        size_t workspace_bytes, void *hip_stream);

/*
 * respec_verify_attention for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, layouts and results as respec_verify_attention (contiguous
 * cache, chain of drafts) without the workspace pair: the scratch of the launch (partial
 * results of cut sequences, the tile prefix, the starting points of the split) lives in a
 * buffer of respec_static_scratch_bytes() bytes (40 MiB) that is part of the library's device
 * image.  Every GPU the library runs on holds its own copy until the process ends.
 *
 *   - A batch whose scratch does not fit (sized for a split of at most 1024 ranges: roughly
 *     G * max_q_per_seq <= 64 at D = 128, B <= about 500,000) is refused with
 *     RESPEC_ERR_WORKSPACE before anything is launched; use respec_verify_attention then.
 *   - The call allocates nothing and frees nothing.  Its first use on a device looks the
 *     buffer's address up (hipGetSymbolAddress); call respec_static_scratch_init() once per
 *     device beforehand where that must not happen inside the call (graph capture).
 *   - All calls on one GPU share the one buffer: calls that overlap on a GPU (two streams,
 *     two host threads) race and give wrong results.  Calls in stream order are fine; nothing
 *     in the buffer has to survive from one call to the next and nothing has to be cleared.
 */
size_t respec_static_scratch_bytes(void);
respec_status_t respec_static_scratch_init(void);
respec_status_t respec_verify_attention_static(const void *q, const void *k_cache, const void *v_cache,
                                               const int32_t *q_indptr, const int64_t *kv_indptr,
                                               void *out, float *lse, int32_t B, int32_t total_q,
                                               int64_t total_kv, int32_t max_q_per_seq,
                                               int32_t max_kv_len, int32_t Hq, int32_t Hkv, int32_t D,
                                               float sm_scale, respec_dtype_t dt, void *hip_stream);

/*
 * The attention of ANOTHER LAYER of the same forward pass.  The target's single forward over the
 * drafted block (Figure 2) runs this attention once per layer with the same sequences: the
 * index arrays, the lengths and every size are those of the previous call, only q, the caches
 * and out (and sm_scale) belong to another layer.  The set-up that a call derives from the
 * index arrays (tile counts, where every wave starts) is then reused instead of being computed
 * again.
 *
 * Contract: `workspace` is the workspace of an earlier respec_verify_attention or
 * respec_verify_attention_tree call (or of a call of this function) on the same stream with the
 * same q_indptr and kv_indptr CONTENTS, B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv,
 * D and dt, and nothing else has written to it since.  tree_mask: NULL for chains, else as in
 * respec_verify_attention_tree.  Everything else as in respec_verify_attention; the result is
 * bit-equal to what a full call on the same arguments gives.  If the contract is broken the
 * output is wrong, but no access leaves the buffers (every index is clamped as in a full call).
 */
respec_status_t respec_verify_attention_next_layer(const void *q, const void *k_cache, const void *v_cache,
                                                   const int32_t *q_indptr, const int64_t *kv_indptr,
                                                   const uint64_t *tree_mask, void *out, float *lse,
                                                   int32_t B, int32_t total_q, int64_t total_kv,
                                                   int32_t max_q_per_seq, int32_t max_kv_len, int32_t Hq,
                                                   int32_t Hkv, int32_t D, float sm_scale, respec_dtype_t dt,
                                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Verify attention over a tree of drafts (Section 4.1: candidate branches, branching factor
 * t, validated in parallel).  As respec_verify_attention, except for which of a sequence's
 * own new tokens a row sees: row i of sequence b (rows in an order in which parents come
 * first, row 0 the root = the last committed token; the R_b new tokens are the last R_b
 * entries of the sequence's KV range, in row order) sees every key before the new tokens
 * and the new token j iff bit j of tree_mask[q_indptr[b]+i] is set (its ancestors and
 * itself; the chain is the mask with bits 0..i).
 *   tree_mask   [total_q] uint64, device memory
 *   max_q_per_seq <= 64 (RESPEC_ERR_UNSUPPORTED otherwise); everything else as above,
 *   the same workspace size.
 */
respec_status_t respec_verify_attention_tree(const void *q, const void *k_cache, const void *v_cache,
                                             const int32_t *q_indptr, const int64_t *kv_indptr,
                                             const uint64_t *tree_mask, void *out, float *lse,
                                             int32_t B, int32_t total_q, int64_t total_kv,
                                             int32_t max_q_per_seq, int32_t max_kv_len, int32_t Hq,
                                             int32_t Hkv, int32_t D, float sm_scale,
                                             respec_dtype_t dt, void *workspace,
                                             size_t workspace_bytes, void *hip_stream);

/*
 * Verify attention over a paged KV cache (the cache the serving side manages while it moves
 * sequences between speculative and plain decoding, Sections 5.1 and 5.2; the paper fixes no
 * layout, this one is the library's).  The result is that of respec_verify_attention (or, with
 * a tree_mask, of respec_verify_attention_tree) on the sequence's tokens taken in order:
 * token j of sequence b lives in slot j % page_size of page
 * page_table[page_indptr[b] + j / page_size].
 *
 *   k_pages, v_pages [num_pages, page_size, Hkv, D] dt, 16-byte aligned
 *   page_indptr   [B+1] int32: the entries of page_table that belong to sequence b
 *   page_table    [page_table_len] int32 page ids in [0, num_pages), token order per sequence;
 *                 a sequence may own more pages than it uses
 *   kv_len        [B] int32: L_b, tokens held by sequence b, the R_b new ones included
 *                 (L_b <= page_size * pages of b; larger values are cut to that)
 *   tree_mask     [total_q] uint64 or NULL (chain)
 *   page_size     a power of two in [16, 1024] (RESPEC_ERR_UNSUPPORTED otherwise)
 *   workspace     respec_verify_attention_workspace_bytes(B, total_q, num_pages*page_size, ...)
 * Everything else as respec_verify_attention.  Page ids outside [0, num_pages) are a caller
 * error; they are clamped, so they cannot cause an access outside the pools.
 */
respec_status_t respec_verify_attention_paged(const void *q, const void *k_pages, const void *v_pages,
                                              const int32_t *q_indptr, const int32_t *page_indptr,
                                              const int32_t *page_table, const int32_t *kv_len,
                                              const uint64_t *tree_mask, void *out, float *lse,
                                              int32_t B, int32_t total_q, int32_t num_pages,
                                              int32_t page_table_len, int32_t page_size,
                                              int32_t max_q_per_seq, int32_t max_kv_len, int32_t Hq,
                                              int32_t Hkv, int32_t D, float sm_scale,
                                              respec_dtype_t dt, void *workspace,
                                              size_t workspace_bytes, void *hip_stream);

/*
 * respec_verify_attention_next_layer for a paged cache: another layer of the same forward,
 * whose K and V pools (k_pages, v_pages) are laid out by the same page table.  Same contract:
 * the workspace is the one of an earlier respec_verify_attention_paged call (or of a call of
 * this function) with the same q_indptr, page_indptr, page_table and kv_len contents and the
 * same sizes, untouched since; the set-up it holds is reused.  Bit-equal to a full call.
 */
respec_status_t respec_verify_attention_paged_next_layer(
    const void *q, const void *k_pages, const void *v_pages, const int32_t *q_indptr,
    const int32_t *page_indptr, const int32_t *page_table, const int32_t *kv_len,
    const uint64_t *tree_mask, void *out, float *lse, int32_t B, int32_t total_q, int32_t num_pages,
    int32_t page_table_len, int32_t page_size, int32_t max_q_per_seq, int32_t max_kv_len, int32_t Hq,
    int32_t Hkv, int32_t D, float sm_scale, respec_dtype_t dt, void *workspace, size_t workspace_bytes,
    void *hip_stream);

/*
 * Commit of a verify step in a paged cache (Section 2.2, "Validation": accepted drafts are
 * kept, the rest of the speculative tokens are dropped; Section 5.2: sequences move between
 * speculative and plain decoding with their cache in place).  Before the call sequence b holds
 * kv_len[b] tokens of which the last R_b are the new ones, row r at position
 * first_new + r (first_new = kv_len[b] - R_b; row 0 is the last committed token).  With
 * n_b = num_accepted[b] accepted nodes, rows path[b, 0] < path[b, 1] < ... (path == NULL: a
 * chain, rows 1..n_b), the K/V of row path[b, j] is moved to position first_new + 1 + j and
 * kv_len[b] becomes first_new + 1 + n_b.  The token drawn last has no K/V yet: the next
 * forward writes it at position kv_len[b].  Slots at or beyond the new length keep whatever
 * they held.  A path entry that is not an increasing row in [j+1, R_b) ends the commit of that
 * sequence at the entries before it.
 *
 *   k_pages, v_pages, page_indptr, page_table, page_size   as respec_verify_attention_paged
 *   kv_len        [B] int32, read and written
 *   path          [B, path_stride] int32 (out_path of respec_tree_rejection_sample) or NULL
 *   num_accepted  [B] int32 (out_num_accepted of either sampler)
 *   Hkv*D*sizeof(element) must be a multiple of 16.
 */
respec_status_t respec_commit_accepted_paged(void *k_pages, void *v_pages, const int32_t *q_indptr,
                                             const int32_t *page_indptr, const int32_t *page_table,
                                             int32_t *kv_len, const int32_t *path, int32_t path_stride,
                                             const int32_t *num_accepted, int32_t B, int32_t total_q,
                                             int32_t max_q_per_seq, int32_t num_pages,
                                             int32_t page_table_len, int32_t page_size, int32_t Hkv,
                                             int32_t D, respec_dtype_t dt, void *hip_stream);

/*
 * Profiling hook (benchmarks only; not for production callers).  One-shot: the calling
 * thread's NEXT attention call (any of the respec_verify_attention* entry points) records
 * `before_main` (if non-NULL) on that call's stream right before its main kernel and
 * `after_main` (if non-NULL) right after it, before the combine kernel; then both are
 * forgotten.  Both are hipEvent_t passed as void*.  Pass NULL, NULL to disarm a hook that was
 * set and not used.  Do not arm it in front of a call that is being captured into a HIP graph.
 * Apart from the knobs below this is the only state the library keeps between calls; it is
 * thread-local.
 */
void respec_profile_mark_main(void *before_main, void *after_main);

/*
 * Test and tuning hook.  The library reads its RESPEC_* environment knobs (forced split
 * widths and kernel forms, used by the tests and by sweeps; none is needed in production)
 * once, at its first call.  A process that changes those variables afterwards calls this to
 * have them read again.  Not thread-safe against calls in flight on other threads.
 */
void respec_reload_knobs(void);

/*
 * Bytes of the optional workspace of respec_rejection_sample.  With a workspace a sequence
 * can be shared by several work-groups (used for batches small enough to leave compute
 * units idle); the workspace holds one small mailbox per sequence through which they
 * exchange partial sums.  Contract: the buffer (device memory, 16-byte aligned) is zero before
 * the first call that uses it; after that the library keeps it consistent from call to call
 * (any B up to the one it was sized for), so it is allocated and cleared once.  Calls that
 * share a workspace must not overlap.  NULL may be passed: one work-group then walks each
 * sequence and nothing else changes.
 *
 * The work-groups that share a sequence wait for one another, so they must all be on the
 * device at the same time: the library never launches more of them than the device has
 * compute units, and the call should have the device to itself (a kernel of another stream
 * that occupies compute units for long can make a wait run out).  A wait that runs out is
 * bounded and reported (out_num_accepted[b] = -1, see respec_rejection_sample); the mailbox
 * of that sequence is then marked unusable and every later call reports -1 for the sequence
 * in that slot until the caller has set the workspace to zero again.  The marks that tell one
 * call's words from another's are 32 bits wide with ten bits for the stage within a call:
 * zero the workspace again before 2^22 (about four million) calls have used it.
 */
size_t respec_rejection_sample_workspace_bytes(int32_t B, int32_t total_q, int32_t V,
                                               respec_dtype_t logits_dt);

/*
 * Speculative rejection sampling with supplied randomness (Section 2.2, Eq. 1 and Eq. 2).
 *
 * Per sequence b with k_b = R_b-1 drafted tokens, for i = 0 .. k_b-1 in order:
 *     p = softmax(target_logits[q_indptr[b]+i, :] / T),  q = softmax(draft_logits[q_indptr[b]-b+i, :] / T)
 *     x = draft_tokens[q_indptr[b]-b+i];  accept iff u_accept[q_indptr[b]-b+i] < min(1, p[x]/q[x])
 * (q[x] == 0 counts as ratio +inf when p[x] > 0, else 0).  At the first rejection i = n the
 * token out_tokens[b,n] is drawn from max(0,p-q)/Z (Eq. 2) and the sequence stops; if all
 * k_b are accepted (or k_b == 0) out_tokens[b,k_b] is drawn from softmax(target row k_b / T).
 * That one draw is an inverse-CDF walk in ascending token id: the first x whose running
 * sum exceeds u_final[b]*Z.  Rows after the first rejection are never used; with a workspace
 * (sequences shared by several work-groups) the row pair right behind a rejected position may
 * have been read ahead of the test, so those rows have to be readable memory of the logits
 * buffers, which they are by the layout above, but may hold anything.
 *
 *   target_logits [total_q, V], row stride ld_t elements (>= V)    logits_dt
 *   draft_logits  [total_q-B, V], row stride ld_d elements (>= V)  logits_dt; may be NULL
 *                 when total_q == B.  Rows start 16-byte aligned for the vector path
 *                 (base and stride); other alignments take a slower scalar path.
 *   draft_tokens  [total_q-B] int32 in [0,V)
 *   q_indptr      [B+1] int32 (the same array verify attention takes)
 *   u_accept      [total_q-B] f32 in [0,1);  u_final [B] f32 in [0,1)
 *   out_tokens    [B, max_k+1] int32 (written): accepted drafts, then the resampled or
 *                 bonus token, then -1
 *   out_num_accepted [B] int32 (written): n_b, the acceptance length (drafts accepted
 *                 before the first rejection)
 *   out_flags     [B] int32 or NULL (written): bit0 = an acceptance test had
 *                 |u - min(1,ratio)| <= 1e-6; bit1 = u_final*Z lay within 1e-6*Z of an edge
 *                 of the chosen token's CDF cell.  Such draws may legitimately differ from
 *                 an exact-arithmetic evaluation.
 *   max_k         host-side upper bound of k_b (row width of out_tokens minus one)
 *   temperature   T > 0, applied to target and drafter logits alike
 *   workspace     NULL, or respec_rejection_sample_workspace_bytes bytes (see there)
 * Errors: RESPEC_ERR_INVALID_ARG / RESPEC_ERR_WORKSPACE before any launch.  If work-groups
 * that share a sequence ever lose each other (a bounded wait runs out: a device fault, a
 * workspace that was not zero at first use, or compute units held by another stream's kernel),
 * out_num_accepted[b] of that sequence is -1 and the workspace has to be zeroed again before
 * its next use (see respec_rejection_sample_workspace_bytes).
 */
respec_status_t respec_rejection_sample(const void *target_logits, const void *draft_logits,
                                        const int32_t *draft_tokens, const int32_t *q_indptr,
                                        const float *u_accept, const float *u_final,
                                        int32_t *out_tokens, int32_t *out_num_accepted,
                                        int32_t *out_flags, int32_t B, int32_t total_q,
                                        int32_t max_k, int32_t V, int64_t ld_t, int64_t ld_d,
                                        float temperature, respec_dtype_t logits_dt,
                                        void *workspace, size_t workspace_bytes,
                                        void *hip_stream);

/*
 * respec_rejection_sample with one temperature per sequence, temperature 0 meaning greedy
 * verification.  The paper runs its tasks at different sampling temperatures (Table 2); a
 * rollout batch can mix them, and evaluation decodes greedily.  For temperature[b] > 0 the
 * sequence is handled exactly as by respec_rejection_sample at that temperature (Section 2.2,
 * Eq. 1 and Eq. 2).  For temperature[b] == 0, the limit of the same rule: softmax(z/T) tends to
 * a point mass on the largest logit, so a drafted token is accepted iff it is the argmax of its
 * target row, the first one that is not is replaced by that argmax, and if all are accepted
 * the bonus token is the argmax of row k_b.  Among equal largest logits the lowest token id is
 * the argmax (and the only one accepted).  A greedy sequence reads target rows 0..n_b only, no
 * drafter logits and no uniforms; its flags are 0.
 *
 *   temperature   [B] f32, device; each finite and >= 0
 *   draft_logits, u_accept   may be NULL when every sequence with drafted tokens is greedy
 *   other arguments as in respec_rejection_sample; there is no workspace (a sequence is
 *   handled by one work-group).
 * Device-side data errors that the host cannot see (a negative or non-finite temperature, a
 * sampled sequence with drafted tokens but draft_logits or u_accept NULL) give
 * out_num_accepted[b] = -1 and out_tokens[b, :] = -1 for that sequence.
 */
respec_status_t respec_rejection_sample_per_seq(const void *target_logits, const void *draft_logits,
                                                const int32_t *draft_tokens, const int32_t *q_indptr,
                                                const float *u_accept, const float *u_final,
                                                const float *temperature, int32_t *out_tokens,
                                                int32_t *out_num_accepted, int32_t *out_flags,
                                                int32_t B, int32_t total_q, int32_t max_k, int32_t V,
                                                int64_t ld_t, int64_t ld_d, respec_dtype_t logits_dt,
                                                void *hip_stream);

/*
 * Rejection sampling over a tree of drafts (Section 4.1: candidate branches with branching
 * factor t validated in parallel; Section 2.2, Eq. 1 and Eq. 2 applied to sibling candidates
 * one after the other).  The paper states the rule for a chain only; this is the reading
 * that keeps the result distributed as the target model when the children of a node are
 * independent draws from the drafter at that node.
 *
 * Sequence b owns rows q_indptr[b] .. q_indptr[b+1]-1, the rows verify attention over a tree
 * takes: row 0 is the root (the last committed token), parent[row] < row is the row's
 * parent within the sequence (-1 for the root).  With cur = 0 and
 *     p = softmax(target_logits[q_indptr[b]+cur, :] / T),  q = softmax(draft_logits[q_indptr[b]+cur, :] / T)
 * the children c of cur are tried in row order: x = node_tokens[q_indptr[b]+c] is accepted
 * iff u_accept[q_indptr[b]+c] < min(1, p[x]/q[x]) (q[x] == 0: ratio +inf if p[x] > 0, else 0);
 * accepted, c becomes cur and the walk goes on from its own rows; rejected, p is replaced by
 * max(0, p-q)/Z (Eq. 2) before the next child is tried.  When no child is left (or cur has
 * none) one token is drawn from the current p by the inverse-CDF walk of
 * respec_rejection_sample with u_final[b].  Rows off the accepted path are never read.
 *
 *   target_logits [total_q, V], row stride ld_t  logits_dt
 *   draft_logits  [total_q, V], row stride ld_d  logits_dt: row r holds the drafter's logits
 *                 for the children of row r (rows of leaves are never read)
 *   node_tokens   [total_q] int32 in [0,V) (the root's entry is never read)
 *   parent        [total_q] int32
 *   u_accept      [total_q] f32 in [0,1) (one per node; the root's is never read)
 *   u_final       [B] f32 in [0,1)
 *   out_tokens    [B, max_depth+1] int32 (written): accepted tokens along the path, then the
 *                 final token, then -1
 *   out_path      [B, max(max_depth,1)] int32 (written): rows of the accepted nodes, then -1
 *   out_num_accepted [B] int32 (written); out_flags [B] or NULL as in respec_rejection_sample
 *                 (bit1 is also set when a residual came out empty and the target was used)
 *   max_q_per_seq host-side bound of the rows of a sequence, <= 64 (RESPEC_ERR_UNSUPPORTED)
 *   max_depth     host-side bound of the depth of any tree (root = depth 0)
 * A chain-shaped tree gives the tokens of respec_rejection_sample bit for bit.
 */
respec_status_t respec_tree_rejection_sample(const void *target_logits, const void *draft_logits,
                                             const int32_t *node_tokens, const int32_t *parent,
                                             const int32_t *q_indptr, const float *u_accept,
                                             const float *u_final, int32_t *out_tokens,
                                             int32_t *out_path, int32_t *out_num_accepted,
                                             int32_t *out_flags, int32_t B, int32_t total_q,
                                             int32_t max_q_per_seq, int32_t max_depth, int32_t V,
                                             int64_t ld_t, int64_t ld_d, float temperature,
                                             respec_dtype_t logits_dt, void *hip_stream);

/*
 * Reward-weighted knowledge distillation of the drafter, per logits row (Section 5.3,
 * "Reward-Weighted Knowledge Distillation"; the update step of Algorithm 1).  For every row r
 *     p = softmax(target_logits[r, :]),  q = softmax(draft_logits[r, :])
 *     row_loss[r] = w_r * KL(p || q) = w_r * sum_x p(x) (log p(x) - log q(x))      (p(x) = 0 terms are 0)
 *     grad_draft_logits[r, x] = w_r * (q(x) - p(x))        (the derivative of row_loss[r] in draft_logits[r, x])
 *     *total_loss = sum_r row_loss[r]
 * w_r = row_weight[r] is the weight w(reward) of the sample the row belongs to; the paper's
 * default w(r) = r, its normalisation and its clipping are the caller's (they are not
 * specified).  Rows with weight 0 are not read; their gradient is written as zero.
 * The rows are the [rows, V] logits the sampler reads.  A row pair is streamed twice (once for
 * its normalisers, once for the gradient) by one work-group; rows are independent.
 *
 *   target_logits, draft_logits [rows, V] logits_dt, row strides ld_t, ld_d elements
 *   row_weight    [rows] f32
 *   grad_draft_logits [rows, V] logits_dt (written; bf16: rounded to nearest even), stride ld_g
 *   row_loss      [rows] f32 (written);  total_loss  [1] f64 or NULL (written)
 *   V * sizeof(element), the strides in bytes and the three base pointers must be multiples of
 *   16 (RESPEC_ERR_UNSUPPORTED otherwise).
 *   workspace     respec_kd_rows_workspace_bytes(rows, V, logits_dt) bytes, 256-byte aligned,
 *                 scratch (nothing to prepare, nothing survives).
 * Asynchronous on hip_stream like every other call; sums are formed in a fixed order, so a call
 * repeated on the same inputs gives the same bits.
 */
size_t respec_kd_rows_workspace_bytes(int32_t rows, int32_t V, respec_dtype_t logits_dt);
respec_status_t respec_kd_rows(const void *target_logits, const void *draft_logits,
                               const float *row_weight, void *grad_draft_logits, float *row_loss,
                               double *total_loss, int32_t rows, int32_t V, int64_t ld_t, int64_t ld_d,
                               int64_t ld_g, respec_dtype_t logits_dt, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/*
 * Debug check of the device-side data that the other entry points cannot report: they clamp
 * every index they derive from q_indptr / kv_indptr (so bad data never causes an access outside
 * the buffers) but then compute something meaningless.  This call checks the arrays of one
 * verify batch (Section 2.2: B sequences, k_b drafted tokens each) and, unlike every other call,
 * WAITS for the result (it synchronises hip_stream).
 *
 * Checked: both index arrays start at 0; every sequence has 1 <= k_b + 1 <= max_q_per_seq rows
 * and k_b + 1 <= L_b <= max_kv_len cached tokens; the last entries equal total_q / total_kv;
 * every drafted token lies in [0, V).
 *
 *   kv_indptr     may be NULL (paged caches: only the rows and the tokens are checked)
 *   draft_tokens  [total_q - B] or NULL (not checked)
 *   workspace     respec_validate_batch_workspace_bytes(B) bytes of device memory, scratch
 * Returns RESPEC_OK, or RESPEC_ERR_INVALID_ARG with respec_last_error() naming the lowest
 * sequence that has a defect and the defect.
 */
size_t respec_validate_batch_workspace_bytes(int32_t B);
respec_status_t respec_validate_batch(const int32_t *q_indptr, const int64_t *kv_indptr,
                                      const int32_t *draft_tokens, int32_t B, int32_t total_q,
                                      int64_t total_kv, int32_t max_q_per_seq, int32_t max_kv_len,
                                      int32_t V, void *workspace, size_t workspace_bytes,
                                      void *hip_stream);

/*
 * The Solver's choice of the draft length for the current active batch size (Section 5.2,
 * "Solver: Offline Profiling Guided Search": configurations are profiled offline per batch
 * size, a performance model predicts the speedup, and at run time the configuration with the
 * best prediction for the observed active batch size is selected).  HOST code: every pointer
 * is a host pointer, nothing touches the GPU.
 *
 * `points` is the offline profile: one entry per (batch size, draft length) that was timed,
 * k = 0 being plain decoding (required).  The model is piecewise linear: for every k the step
 * time and the emitted tokens per sequence at `active_batch` are interpolated between the
 * profiled batch sizes (the end values hold outside their range).  The choice minimises the
 * cost per produced token of Eq. 4, (k C_q + k C_p / alpha) / (r k), with measured quantities
 * in the place of its symbols: k C_p / alpha is the verify step's time at (batch, k), r k the
 * tokens a step emits per sequence, C_q = draft_us_fixed + draft_us_per_seq * active_batch the
 * time of one drafter step:
 *     cost(k) = (k * C_q + step_us(batch, k)) / emitted_per_seq(batch, k).
 * Ties go to the smaller k.
 *
 *   best_k    (written) the chosen draft length; 0 = speculation off
 *   speedup   (written, or NULL) cost(0) / cost(best_k), >= 1
 *   cost_us   (written, or NULL) cost(best_k)
 * RESPEC_ERR_INVALID_ARG: empty table, no k = 0 point, a non-positive or non-finite entry.
 */
typedef struct {
    int32_t batch;           /* sequences in the profiled batch */
    int32_t k;               /* drafted tokens per sequence, 0 = plain decoding */
    double step_us;          /* time of one target step at (batch, k) */
    double emitted_per_seq;  /* tokens emitted per sequence and step (1 for k = 0) */
} respec_profile_point_t;

respec_status_t respec_solver_pick(const respec_profile_point_t *points, int32_t n_points,
                                   int32_t active_batch, double draft_us_fixed,
                                   double draft_us_per_seq, int32_t *best_k, double *speedup,
                                   double *cost_us);

#ifdef __cplusplus
}
#endif
#endif /* RESPEC_H */
