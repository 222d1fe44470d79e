/*
 * specgbv.h -- C ABI of the MI355X SpecTr-GBV verification library (libspecgbv.so).
 *
 * One call verifies, for a batch of independent prefixes, K i.i.d. draft blocks
 * of length L against the target model: paper Section 4.2, Algorithm 1
 * ("SpecTr-GBV"), with the sub-block and whole-block acceptance probabilities
 * of Eq. (hik) and Eq. (hLk) and the residual distribution of Eq. (pres).
 *
 * All logits/tokens/outputs/workspace pointers are DEVICE pointers; the library
 * allocates no device memory, never synchronises the stream (except
 * specgbv_read_intermediates) and keeps no state between calls: the same inputs
 * with the same (rng_seed, rng_offset) give the same outputs.
 *
 * Row convention.  For prefix b and draft k, target row r is q(.|x_k^r), the
 * target distribution after the first r draft tokens (r = 0..L; row L serves
 * the bonus token), draft row r is p(.|x_k^r) (r = 0..L-1) and
 * draft_tokens[b,k,r] = x_k^(r+1) is the token drawn from draft row r.
 * Distributions are softmax(logits / temperature) for both models.
 *
 * Randomness.  Uniforms are Philox4x32-10 outputs with key = rng_seed and
 * counter = (rng_offset low, rng_offset high, b, slot); slot = k*L + (i-1) for
 * the acceptance test of sub-block length i of draft k, slot = K*L for the
 * final token; u = (word0 >> 8) * 2^-24.  A call consumes exactly these
 * counters; advance rng_offset by one per call.
 */
#ifndef SPECGBV_H
#define SPECGBV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPECGBV_OK = 0,
    SPECGBV_EINVAL = 1,        /* null pointer, non-positive size, bad temperature, ...   */
    SPECGBV_EUNSUPPORTED = 2,  /* valid request outside the implemented limits            */
    SPECGBV_EWORKSPACE = 3,    /* workspace null, misaligned or smaller than required     */
    SPECGBV_EHIP = 4           /* a HIP runtime call failed (launch, event record, copy)  */
} specgbv_status;

typedef enum {
    SPECGBV_F32 = 0,           /* IEEE float32 logits                                      */
    SPECGBV_BF16 = 1           /* bfloat16 logits, widened to float32 in the kernels       */
} specgbv_dtype;

/* Kernel schedule.  AUTO picks by shape; the other values force one schedule (for tests
 * and measurements) and fail with SPECGBV_EUNSUPPORTED if the shape does not allow it. */
typedef enum {
    SPECGBV_ALGO_AUTO = 0,
    SPECGBV_ALGO_SPLIT = 1,    /* statistics pass, then a second pass for the sums of Eq. (hik) */
    SPECGBV_ALGO_CHAIN = 2     /* one workgroup per (prefix, draft) keeps each row pair on chip  */
} specgbv_algo;

/* Limits (checked; violations return SPECGBV_EUNSUPPORTED). */
#define SPECGBV_MAX_K 64
#define SPECGBV_MAX_L 62

/*
 * Bytes of device workspace specgbv_verify needs for this shape (0 if the shape is
 * invalid).  The workspace must be 256-byte aligned; its contents need not be
 * initialised and are overwritten by every call.
 */
size_t specgbv_workspace_bytes(int batch, int K, int L, int V, specgbv_dtype dtype);

/*
 * Multi-draft greedy block verification (Algorithm 1; Eq. (hik), Eq. (hLk), Eq. (pres)).
 *
 *   target_logits      device, [batch, K, L+1, V], dense, V fastest
 *   draft_logits       device, [batch, K, L,   V], dense, V fastest.  Logits may be -inf
 *                      (masked vocabulary entries: probability 0, residual weight 0) but
 *                      not +inf or NaN, and every row needs at least one finite entry; a
 *                      drafted token whose target logit is -inf makes its block and every
 *                      longer one unacceptable (h = 0)
 *   draft_tokens       device, [batch, K, L] int32, each in [0, V) (not checked on device
 *                      beyond clamping the gather index; out-of-range tokens give
 *                      meaningless but memory-safe results)
 *   K, L, V, batch     >= 1 (batch may be 0: nothing is launched); K <= SPECGBV_MAX_K,
 *                      L <= SPECGBV_MAX_L
 *   dtype              element type of both logits tensors
 *   temperature        > 0 and finite; applied to both models
 *   rng_seed/offset    Philox key and call counter (see above)
 *   accepted_len       device out, [batch] int32: tau in [0, L]
 *   accepted_draft_idx device out, [batch] int32: index f of the draft whose first tau
 *                      tokens were accepted, -1 when tau = 0
 *   out_tokens         device out, [batch, L+1] int32: the tau accepted tokens, then the
 *                      final token y (residual draw of Eq. (pres) when tau < L, a draw from
 *                      target row L of draft f when tau = L), then -1 padding
 *   workspace          device, >= specgbv_workspace_bytes(...) bytes, 256-byte aligned
 *   hip_stream         hipStream_t (NULL = default stream); all work is enqueued on it and
 *                      the call returns without waiting
 *
 * Readings where the paper is silent: 0/0 in Eq. (hik) is 1; acceptance probabilities are
 * clamped to [0,1]; the final token is the first id whose running weight sum exceeds
 * u * total; if every residual weight is zero the token is drawn from target row tau; the
 * tau = 0 residual uses rows 0 of draft 0.
 *
 * Errors are detected on the host before anything is launched; on error nothing is
 * written and specgbv_last_error() describes the cause.
 *
 * Environment (read at every call, meant for tests): SPECGBV_EXCESS_POLLS = how often a workgroup of the
 * final-token kernel looks for a partial sum another workgroup of its prefix owes before it takes that sum
 * itself (small batches; default 1024, 0 = never wait).  The results do not depend on it.
 */
specgbv_status specgbv_verify(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * specgbv_verify for callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: same arguments, semantics and outputs as specgbv_verify
 * (default schedule), without the workspace.  The kernels' scratch memory (row statistics, the sums of Eq. (hik),
 * partial sums and arrival counters of the final-token search) lives in a buffer of
 * SPECGBV_STATIC_SCRATCH_BYTES built into the library's device image: every GPU the library runs on holds its own
 * copy until the process ends.  The call allocates and frees nothing.
 *
 *   - A shape with specgbv_workspace_bytes(batch, K, L, V, dtype) > SPECGBV_STATIC_SCRATCH_BYTES is refused with
 *     SPECGBV_EUNSUPPORTED before anything is launched.
 *   - All calls on one GPU share that GPU's buffer: two calls that overlap in time on one GPU (different streams,
 *     or different host threads) race and give undefined results; calls on one stream are ordered and safe.  The
 *     buffer keeps the previous call's contents; every call rewrites what it reads (the arrival counters are
 *     cleared by the call's first kernel), so no clearing is needed between calls.
 *   - The buffer's address on a GPU is looked up on the first call with that GPU current (not an allocation, but
 *     make that first call outside a graph capture).
 *   - specgbv_read_intermediates and specgbv_workspace_carry need a caller-owned workspace and do not apply.
 */
#define SPECGBV_STATIC_SCRATCH_BYTES (8u << 20)
specgbv_status specgbv_verify_static(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens, void *hip_stream);

/*
 * Comparison verifiers on the same inputs (paper Section 3, the methods SpecTr-GBV is measured against):
 * SpecTr's K-SEQ rule (Section 3.2) on the first `ndrafts` of the K drafts; ndrafts = 1 is token-level
 * speculative decoding (Section 3.1: accept x with probability min{1, q/p}, residual norm(max{q - p, 0})).
 *
 * Position by position, the candidates are the tokens of the drafts still retained (those that agree with
 * everything accepted so far), in draft order; candidate x is accepted with probability
 * min{1, q(x) / (rho p(x))}; the first accepted one is emitted and the drafts carrying it stay retained; if none
 * is accepted the replacement is drawn from (q - rho min{p, q/rho}) / (1 - rho beta(rho)) and the iteration ends;
 * after L accepted positions a bonus token is drawn from target row L.  rho in [1, k] solves
 * 1 - (1 - beta(rho))^k = rho beta(rho), beta(rho) = sum_x min{p(x), q(x)/rho}, with k the number of drafts
 * retained at that position (K at the first one; this reading keeps the output distributed as the target).
 * The distributions of a position are read from the rows of the retained draft of lowest index.
 *
 * Arguments, outputs, workspace (specgbv_workspace_bytes of the same shape) and error behaviour as specgbv_verify;
 * accepted_draft_idx receives the retained draft of lowest index (-1 when nothing was accepted).  Uniforms:
 * Philox slot j*L + (i-1) for draft j's test at position i, slot K*L for the final token.
 */
specgbv_status specgbv_verify_kseq(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset, int ndrafts,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/* HOST buffers receiving the intermediates of the last specgbv_verify_kseq call that used a workspace (any
 * pointer may be NULL); Section 3.2. */
typedef struct specgbv_kseq_intermediates {
    double *rho_all;     /* [batch, K, L]  rho of row r of draft j, solved for the number of drafts sharing   */
                         /*                draft j's first r tokens (drafts beyond ndrafts: not written)     */
    double *beta_all;    /* [batch, K, L]  beta(rho) there                                                    */
    double *accept;      /* [batch, K, L]  acceptance probability of draft j's token at position r+1          */
    double *eta;         /* [batch, K, L]  uniform of that test                                               */
    int32_t *state;      /* [batch, K, L]  1 where the test was performed                                     */
    int32_t *retained;   /* [batch, L]     drafts retained when position r+1 was verified (0: not reached)    */
    int32_t *lead;       /* [batch, L]     the lowest of them (-1: not reached)                               */
    double *res_norm;    /* [batch] total weight the final token was drawn from                               */
    double *u_final;     /* [batch] */
    double *margin;      /* [batch] */
} specgbv_kseq_intermediates;

/* Copies them to host memory and waits for the copies (debug/parity aid). */
specgbv_status specgbv_read_kseq_intermediates(
    const void *workspace, size_t workspace_bytes, int batch, int K, int L, int V,
    const specgbv_kseq_intermediates *host_out, void *hip_stream);

#define SPECGBV_MAX_PENDING 16  /* pending distribution modifications applied on the fly at most */

/* Extra controls for specgbv_verify_ex; zero-initialise for the defaults. */
typedef struct specgbv_options {
    int32_t algo;              /* specgbv_algo                                              */
    int32_t pending_levels;    /* see pending_carry_log_nu                                  */
    void *ev_main_start;       /* hipEvent_t or NULL: recorded on the stream immediately    */
    void *ev_main_stop;        /*   before / after the vocabulary-streaming kernels that    */
                               /*   compute the statistics and the sums of Eq. (hik) for    */
                               /*   every row (the chain schedule's small follow-up kernel  */
                               /*   for the rare rows whose sum is taken a second time and  */
                               /*   the final-token kernel come after the stop event)       */
    /*
     * Pending distribution modifications (Algorithm 2) applied on the fly: both pointers NULL (none) or
     * both device pointers to pending_levels arrays of [batch] values, innermost level first
     * (pending_levels = 0 with pointers given means 1; at most SPECGBV_MAX_PENDING).  Level l makes the
     * first pending_count[l][b] rows of every draft of prefix b the distribution q_new of Algorithm 2,
     * computed from the rows as the levels before it left them and from the same draft rows, with the
     * block ratio starting from exp(pending_carry_log_nu[l][b]); nothing is written out, and the
     * outputs are those of specgbv_modify_target applied level by level followed by a verification
     * of its rows.  One level is what the previous iteration left in its workspace
     * (specgbv_workspace_carry; the pointers may point into the workspace passed to this call: they
     * are read before the new values are written); several levels arise when an iteration ends
     * before the previous modification's rows are used up (Algorithm 3 updates q in place).
     * SPECGBV_ALGO_AUTO takes the two-pass schedule; SPECGBV_ALGO_CHAIN applies the levels by extra
     * sweeps over the on-chip row pair (rows that do not fit on chip are rejected), which is faster
     * while few rows are modified.  A modified row whose weights are all zero stays as it was.
     */
    const double *pending_carry_log_nu;   /* device, [pending_levels][batch] */
    const int32_t *pending_count;         /* device, [pending_levels][batch], values below 0 or above L are clamped */
    /*
     * Or (instead of the two pointers above, which must then be NULL): the whole bookkeeping of
     * Algorithm 3 on the device.  pending_state is a device buffer of
     * specgbv_pending_state_bytes(batch) bytes, all zero before the first iteration of a prefix; the
     * call applies the modifications it holds and then updates it in place: every level's ratio is
     * moved along the tokens this iteration emits and its count reduced (specgbv_carry_advance),
     * levels whose rows are used up are dropped, and the modification this iteration creates is
     * appended.  Needs L - 1 <= SPECGBV_MAX_PENDING.  Calls on one state must not overlap.
     */
    void *pending_state;
    /*
     * Nonzero: the caller states that rows 0 of the K drafts of a prefix are copies of one another in both
     * tensors (they are in Algorithm 3: the K drafts of an iteration extend the same prefix, so
     * position 0 of every draft is conditioned on that prefix alone; Section 4).  The chain schedule then reads
     * rows 0 once per prefix (the copy of draft 0) instead of once per draft; other schedules, and calls
     * with pending modifications, ignore the hint.  With rows 0 that differ the results are those of
     * draft 0's rows 0 used for every draft's statistics of position 0.
     */
    int32_t shared_row0;
    int32_t reserved;          /* 0 */
} specgbv_options;

/* specgbv_verify with explicit options (options == NULL means defaults). */
specgbv_status specgbv_verify_ex(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream,
    const specgbv_options *options);

/* Bytes of the pending_state buffer of specgbv_options for `batch` prefixes (0 if batch < 0): SPECGBV_MAX_PENDING
 * carried ratios (float64) and row counts (int32) per prefix, level-major.  Section 4.2, Algorithms 2 and 3. */
size_t specgbv_pending_state_bytes(int batch);

/*
 * HOST buffers receiving the intermediates of the most recent call that used a
 * workspace (any pointer may be NULL).  Arrays indexed by the sub-block length
 * i = 1..L store entry i at position i-1.
 */
typedef struct specgbv_intermediates {
    double *lse_q;       /* [batch, K, L]  ln sum_x exp(z_q/T) of target rows 0..L-1        */
    double *lse_p;       /* [batch, K, L]  same for the draft rows                          */
    double *log_nu;      /* [batch, K, L]  ln nu_i, the block likelihood ratio Q_i / P_i    */
    double *log_P;       /* [batch, K, L]  ln P_i, the draft probability of the block       */
    double *s;           /* [batch, K, L]  vocabulary sum of Eq. (hik) divided by q(x^i),   */
                         /*                at position i (i = 1..L-1; position 0 is NaN)    */
    double *h;           /* [batch, K, L]  acceptance probability of sub-block length i     */
    double *eta;         /* [batch, K, L]  uniform of that test                             */
    int32_t *state;      /* [batch, K, L]  0 never reached, 1 tested, 2 skipped (block in H) */
    double *res_norm;    /* [batch] total weight the final token was drawn from (weights    */
                         /*         are q[x] * max(1 - p[x]/(nu q[x]), 0)^K, or q[x])        */
    double *u_final;     /* [batch] uniform of the final token                              */
    double *margin;      /* [batch] distance of u*total to the nearer end of the drawn      */
                         /*         token's CDF interval, divided by total                  */
    int32_t *fallback;   /* [batch] 1 if all residual weights were zero                     */
    double *carry_log_nu;   /* [batch] ln [q(t^tau, y) / p(t^tau, y)] relative to the prefix: the */
                            /*         block ratio Algorithm 2 starts from (0 when tau = L)    */
    int32_t *modify_count;  /* [batch] L - tau - 1 rows Algorithm 2 modifies next (0 if tau = L) */
} specgbv_intermediates;

/*
 * Copies the intermediates left in `workspace` by the last specgbv_verify[_ex] call with
 * the same (batch, K, L) to host memory and waits for the copies (this is the only
 * function that synchronises the stream).  Debug/parity aid, not part of the hot path.
 */
specgbv_status specgbv_read_intermediates(
    const void *workspace, size_t workspace_bytes, int batch, int K, int L, int V,
    specgbv_dtype dtype, const specgbv_intermediates *host_out, void *hip_stream);

/*
 * Device pointers, inside `workspace`, of the two per-prefix values every specgbv_verify[_ex]
 * call leaves for the distribution modification of the next decoding iteration
 * (Algorithm 2; Section 4.2): carry_log_nu [batch] float64 and modify_count [batch] int32, as
 * described in specgbv_intermediates.  They stay valid until the next call that uses the
 * workspace; pass them to specgbv_modify_target on the same stream, or copy them out.
 * (batch, K, L, V) must be those of the verification call.  Host-side arithmetic only.
 */
specgbv_status specgbv_workspace_carry(
    void *workspace, size_t workspace_bytes, int batch, int K, int L, int V,
    double **carry_log_nu, int32_t **modify_count);

/*
 * Distribution modification (Algorithm 2, Section 4.2) for the drafts of the NEXT iteration.
 *
 * After an iteration accepted t^tau and drew y, the first count = L - tau - 1 target rows of
 * every new draft are replaced by
 *     q_new[x] = w[x] / sum_x w[x],   w[x] = q_r[x] * max(1 - p_r[x] / (nu_r q_r[x]), 0)^K
 * (Algorithm 2 with numerator and normaliser divided by the joint probability of the
 * conditioning block, the per-token form of Eq. (pres)), where
 * nu_r = exp(carry_log_nu) * prod_{j<r} q_j[x^(j+1)] / p_j[x^(j+1)] continues the previous
 * iteration's block ratio along the new draft's own tokens with the ORIGINAL target
 * probabilities.  Rows r >= count are left as q_r.  If every weight of a row is zero the row
 * is left as q_r (same reading as for the residual of Eq. (pres)).
 *
 *   target_logits   device, [batch, K, M + bonus_row, V]: target rows r = 0..M-1 of the new
 *                   drafts (row r is conditioned on the new prefix and the draft's first r
 *                   tokens) and, with bonus_row = 1, row M, which Algorithm 2 never modifies
 *                   (the bonus-token row of the next verification)
 *   draft_logits    device, [batch, K, M, V]: the draft rows the tokens were drawn from
 *   draft_tokens    device, [batch, K, M] int32, each in [0, V)
 *   K, M, V, batch  K, M, V >= 1, batch >= 0; K <= SPECGBV_MAX_K, M <= SPECGBV_MAX_L; bonus_row is
 *                   0 or 1
 *   dtype, temperature   as in specgbv_verify
 *   carry_log_nu    device, [batch] float64; modify_count device, [batch] int32, clamped to
 *                   [0, M] (both as left by the previous specgbv_verify call)
 *   out_logq        device out, [batch, K, M + bonus_row, V] float32: natural logarithm of the
 *                   distribution to verify row r against (q_new for r < count, q otherwise;
 *                   -inf where the probability is 0).  Being normalised log-probabilities the
 *                   rows can be handed to specgbv_verify as float32 logits at temperature 1
 *                   (with M = L and bonus_row = 1 the tensor has the shape it expects).
 *   out_logp        device out or NULL, [batch, K, M, V] float32: ln p_r, so that both models
 *                   can be passed on at temperature 1
 *   norm_out        device out or NULL, [batch, K, M] float64: sum_x w[x] of modified rows
 *                   (1 for unmodified rows and for rows whose weights were all zero)
 *   fallback_out    device out or NULL, [batch, K, M] int32: 1 where all weights were zero
 *   workspace       device, >= specgbv_modify_workspace_bytes(batch, K, M, bonus_row) bytes,
 *                   256-byte aligned, contents need not be initialised (per-row statistics);
 *                   it must not be the verification workspace that carry_log_nu and
 *                   modify_count point into
 *   hip_stream      all work is enqueued on it; the call does not wait
 *
 * Errors are detected on the host before anything is launched.
 */
specgbv_status specgbv_modify_target(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int M, int bonus_row, int V, int batch, specgbv_dtype dtype, float temperature,
    const double *carry_log_nu, const int32_t *modify_count,
    float *out_logq, float *out_logp, double *norm_out, int32_t *fallback_out,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace specgbv_modify_target needs (0 if the shape is invalid). */
size_t specgbv_modify_workspace_bytes(int batch, int K, int M, int bonus_row);

/*
 * Book-keeping of Algorithm 3's "q <- DistributionModification(q, p, L, t^tau, y)" over several
 * iterations.  The statement updates q in place, so a modification made after iteration n is
 * still in force for its remaining rows when iteration n+1 emits fewer tokens than it has rows,
 * and iteration n+1's own modification then applies ON TOP of it.  A prefix therefore carries up
 * to L-1 pending modifications (carry_log_nu, modify_count), innermost (oldest) first; the rows
 * to verify are obtained by applying them in that order with specgbv_modify_target (the first
 * on the models' logits, each later one on the previous call's out_logq / out_logp at
 * temperature 1), and after the verification every pending one is advanced by this function:
 *
 *   tau = accepted_len[b], f = max(accepted_draft_idx[b], 0),
 *   e_j = draft_tokens[b, f, j] for j < tau, e_tau = out_tokens[b, tau]      (the emitted tokens)
 *   if modify_count[b] > tau + 1 and tau < M:
 *       carry_log_nu[b] += sum_{j=0..tau} ln q_j[e_j] - ln p_j[e_j],   modify_count[b] -= tau + 1
 *   else modify_count[b] = 0                                   (the modification has expired)
 *
 * with q_j = softmax(rows_q[b, f, j, :] / temperature), the distribution THIS pending
 * modification modifies (the models' target rows for the innermost one, the out_logq of the
 * call below it otherwise), and p_j = softmax(rows_p[b, f, j, :] / temperature).  The newest
 * modification is the pair the verification leaves in its workspace (specgbv_workspace_carry;
 * copy it out before the workspace is reused).
 *
 *   rows_q        device, [batch, K, M + bonus_row, V];  rows_p  device, [batch, K, M, V]
 *   draft_tokens  device, [batch, K, M];  accepted_len, accepted_draft_idx  device, [batch];
 *   out_tokens    device, [batch, M + 1]  (all three as written by specgbv_verify with L = M)
 *   carry_log_nu  device in/out, [batch] float64;  modify_count  device in/out, [batch] int32
 *   workspace     device, >= specgbv_carry_workspace_bytes(batch, M) bytes, 256-byte aligned
 *   batch <= 65535; limits and error behaviour as for specgbv_modify_target
 */
specgbv_status specgbv_carry_advance(
    const void *rows_q, const void *rows_p, const int32_t *draft_tokens,
    const int32_t *accepted_len, const int32_t *accepted_draft_idx, const int32_t *out_tokens,
    int K, int M, int bonus_row, int V, int batch, specgbv_dtype dtype, float temperature,
    double *carry_log_nu, int32_t *modify_count, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace specgbv_carry_advance needs (0 if the shape is invalid). */
size_t specgbv_carry_workspace_bytes(int batch, int M);

/*
 * Draft-side sampling (Algorithm 3, the step "sample x_1^L, ..., x_K^L ~ p i.i.d."): one token
 * per row from softmax(logits[row, :] / temperature).  Called once per draft position with the
 * batch * K draft rows of that position, it draws the K i.i.d. continuations of every prefix.
 *
 * The token of row r is the first id whose running weight sum exceeds u * total (the rule of
 * the final token of specgbv_verify), with u the Philox4x32-10 uniform of key = rng_seed and
 * counter = (rng_offset low, rng_offset high, r, 2^31 + position): slots at or above 2^31 are
 * never used by specgbv_verify, so one (seed, offset) pair can serve a whole decoding iteration.
 *
 *   logits       device, [rows, V], dense; -inf entries have probability 0
 *   rows, V      rows >= 0 (0: nothing is launched), 1 <= V <= 1048576
 *   position     draft position the rows belong to, below 2^31 (selects the Philox slot)
 *   out_tokens   device out, [rows] int32
 *   workspace    device, >= specgbv_sample_workspace_bytes(rows, V) bytes, 256-byte aligned,
 *                contents need not be initialised
 */
specgbv_status specgbv_sample_tokens(
    const void *logits, int rows, int V, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset, uint32_t position, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace specgbv_sample_tokens needs (0 if the shape is invalid). */
size_t specgbv_sample_workspace_bytes(int rows, int V);

/*
 * Copies to HOST buffers (either may be NULL) the uniforms [rows] and the inverse-CDF margins
 * [rows] (distance of u * total to the nearer end of the drawn token's interval, over total)
 * of the last specgbv_sample_tokens call that used `workspace`, and waits for the copies.
 * Debug/parity aid.
 */
specgbv_status specgbv_read_sample_intermediates(
    const void *workspace, size_t workspace_bytes, int rows, int V,
    double *u_host, double *margin_host, void *hip_stream);

/* Message of the last failing call made by this thread ("" if none); static storage. */
const char *specgbv_last_error(void);

/* Library version string, static storage. */
const char *specgbv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECGBV_H */
