/*
 * specgbv_oracle.c -- plain CPU float64 oracle for SpecTr-GBV verification.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct reference
 * that the GPU library is compared against.  It shares no code with the HIP
 * path; only tests, the smoke check and the benchmark's cpu_baseline leg may
 * link or load it.
 *
 * What it computes (paper, Section 4.2): Algorithm 1 "SpecTr-GBV" with the
 * acceptance probabilities of Eq. (hik) [sub-block] and Eq. (hLk) [whole
 * block] and the residual distribution of Eq. (pres), for a batch of
 * independent prefixes, Algorithm 2 "Distribution Modification" (the
 * target distribution of the first L - tau - 1 positions of the next
 * iteration), and the drafting step of Algorithm 3 (one token per draft row).  Everything is written in the order and notation of the paper;
 * there is no blocking, fusion or reordering.
 *
 * Notation.  For one prefix and one draft k: row r (0-based) of the target
 * (draft) logits is the conditional distribution q(.|x^r) (p(.|x^r)), i.e. the
 * one that draft token x^(r+1) = tokens[r] was drawn from; the target has one
 * more row (r = L) used for the bonus token.  With q_r = softmax(z_q/T) and
 * p_r = softmax(z_p/T),
 *     P_i = prod_{j<=i} p_{j-1}[x^(j)],   Q_i likewise,   nu_i = Q_i / P_i
 * (nu_i is the block likelihood ratio of greedy block verification,
 * Section 3.3).  Arrays of shape [.., L] that are indexed by the sub-block
 * length i = 1..L store entry i at position i-1.
 *
 * Rescaled form of the acceptance probabilities.  Eq. (hik) and Eq. (hLk) are
 * written in the paper with joint block probabilities p(x^i), q(x^i), which
 * underflow for realistic L and V.  Dividing numerator and denominator by
 * P_i gives the algebraically identical
 *     s_i  = sum_x q_i[x] * max(1 - p_i[x] / (nu_i q_i[x]), 0)^K
 *     g_i  = max(1 - 1/nu_i, 0)^K
 *     c_K(P) = (1 - (1-P)^K) / P
 *     h_ik = nu_i (s_i - g_i) / (c_K(P_i) - nu_i (1 - s_i)),   i < L
 *     h_Lk = nu_L (1 - g_L) / c_K(P_L)
 * which is what this file evaluates (tests check it against the literal
 * equations in exact rational arithmetic).  For nu_i > 1, where s_i - g_i cancels,
 * Eq. (hik) is evaluated through the equivalent sum of non-negative terms described at
 * specgbv_oracle_ot_excess.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - uniforms come from Philox4x32-10 (Salmon et al., SC'11) with
 *     key = seed, counter = (offset_lo, offset_hi, prefix index, slot),
 *     slot = k*L + (i-1) for the test of sub-block i of draft k and K*L for the
 *     final token; u = (word0 >> 8) * 2^-24;
 *   - the final token is drawn by inverse CDF in token-id order,
 *     y = min{ j : sum_{x<=j} w_x > u * sum_x w_x };
 *   - 0/0 in Eq. (hik) is read as its limit 1; h is clamped to [0,1];
 *   - if every residual weight is zero the token is drawn from q_tau itself;
 *   - tau = 0 uses row 0 of draft 0 and reports draft index -1.
 *
 * Parity status: every function is pinned by tests/test_oracle_*.py
 * (closed forms, exact-rational enumeration of Algorithm 1, K=1 reduction to
 * greedy block verification, library log-softmax, published Philox
 * known-answer vectors).
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
#define ORACLE_F64 2      /* float64 rows: lets one oracle result (log-probabilities) feed another exactly */

/* ------------------------------------------------------------------ Philox */

/* One Philox4x32 round: two 32x32->64 multiplies, then the permutation and
 * key injection of the published S-P network. */
static void philox_round(uint32_t c[4], const uint32_t k[2])
{
    const uint64_t m0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t m1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t hi0 = (uint32_t)(m0 >> 32), lo0 = (uint32_t)m0;
    const uint32_t hi1 = (uint32_t)(m1 >> 32), lo1 = (uint32_t)m1;
    const uint32_t n0 = hi1 ^ c[1] ^ k[0];
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c[3] ^ k[1];
    const uint32_t n3 = lo0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

/* Philox4x32-10: ten rounds, the key advanced by the Weyl constants between
 * rounds. */
void specgbv_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                                  uint32_t out[4])
{
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    uint32_t k[2] = { key[0], key[1] };
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k[0] += 0x9E3779B9u; k[1] += 0xBB67AE85u; }
        philox_round(c, k);
    }
    memcpy(out, c, sizeof c);
}

/* The uniform of one test: 24 random bits, exactly representable in float32
 * and float64, in [0,1). */
double specgbv_oracle_uniform(uint64_t seed, uint64_t offset, uint32_t prefix,
                              uint32_t slot)
{
    const uint32_t ctr[4] = { (uint32_t)offset, (uint32_t)(offset >> 32), prefix, slot };
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    specgbv_oracle_philox4x32_10(ctr, key, out);
    return (double)(out[0] >> 8) * (1.0 / 16777216.0);
}

/* ------------------------------------------------------- input conversions */

static double bf16_to_double(uint16_t h)
{
    const uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static void load_row(const void *base, int dtype, size_t row, int V, double *z)
{
    if (dtype == ORACLE_BF16) {
        const uint16_t *p = (const uint16_t *)base + row * (size_t)V;
        for (int x = 0; x < V; ++x) z[x] = bf16_to_double(p[x]);
    } else if (dtype == ORACLE_F64) {
        memcpy(z, (const double *)base + row * (size_t)V, sizeof(double) * (size_t)V);
    } else {
        const float *p = (const float *)base + row * (size_t)V;
        for (int x = 0; x < V; ++x) z[x] = (double)p[x];
    }
}

/* ----------------------------------------------------------------- softmax */

/* log softmax(z / T): out[x] = z[x]/T - lse, lse = log sum_x exp(z[x]/T).
 * Returns lse. */
double specgbv_oracle_log_softmax(const double *z, int V, double T, double *out)
{
    double m = -INFINITY;
    for (int x = 0; x < V; ++x) {
        out[x] = z[x] / T;
        if (out[x] > m) m = out[x];
    }
    double sum = 0.0;
    for (int x = 0; x < V; ++x) sum += exp(out[x] - m);
    const double lse = m + log(sum);
    for (int x = 0; x < V; ++x) out[x] -= lse;
    return lse;
}

/* ----------------------------------------------------- Eq. (hik) / (hLk) */

static double ipow(double t, int K)
{
    double r = 1.0;
    for (int j = 0; j < K; ++j) r *= t;
    return r;
}

/* One term of the vocabulary sums of Eq. (hik) and Eq. (pres) after dividing
 * by q(x^i):  q[x] * (1 - min{ p[x] / (nu q[x]), 1 })^K. */
static double ot_term(double lq, double lp, double log_nu, int K)
{
    const double ratio = exp(lp - lq - log_nu);
    const double t = 1.0 - (ratio < 1.0 ? ratio : 1.0);
    return exp(lq) * ipow(t, K);
}

/* s = sum_x q[x] * max(1 - p[x]/(nu q[x]), 0)^K, plain left-to-right. */
double specgbv_oracle_ot_sum(const double *lq, const double *lp, int V,
                             double log_nu, int K)
{
    double s = 0.0;
    for (int x = 0; x < V; ++x) s += ot_term(lq[x], lp[x], log_nu, K);
    return s;
}

/* c_K(P) = (1 - (1-P)^K) / P, the probability that at least one of K i.i.d.
 * drafts equals a block of draft probability P, divided by P. */
static double c_K(double logP, int K)
{
    const double P = exp(logP);
    if (P <= 0.0) return (double)K;           /* limit P -> 0 */
    if (P >= 1.0) return 1.0;
    return -expm1((double)K * log1p(-P)) / P;
}

static double g_K(double log_nu, int K)
{
    const double t = 1.0 - exp(-log_nu);      /* 1 - min{P/Q, 1} */
    return t > 0.0 ? ipow(t, K) : 0.0;
}

static double clamp01(double h)
{
    if (!(h > 0.0)) return 0.0;
    return h < 1.0 ? h : 1.0;
}

/* Eq. (hik), sub-block of length i < L, rescaled by P_i. */
double specgbv_oracle_h_sub(double log_nu, double logP, double s, int K)
{
    const double nu = exp(log_nu);
    const double num = nu * (s - g_K(log_nu, K));
    const double den = c_K(logP, K) - nu * (1.0 - s);
    if (!(den > 0.0)) return 1.0;             /* 0/0: limit is 1 */
    return clamp01(num / den);
}

/*
 * Eq. (hik) for nu > 1 without the difference s - g.
 *
 * For nu > 1 the numerator nu (s - g) of the rescaled Eq. (hik) subtracts two numbers that agree
 * to about 1/nu^2: in float64 the difference is already wrong in the sixth digit at nu = 1e5 and
 * meaningless beyond 1e8, although the quotient has a perfectly finite limit.  Both sums of the
 * equation are expectations under q of the convex function phi(rho) = max(1 - rho/nu, 0)^K of
 * the ratio rho = p[x]/q[x], whose mean is 1:  s = E_q phi(rho),  g = phi(1) = phi(E_q rho).
 * Adding the vanishing term -phi'(1) E_q[rho - 1] gives a sum of non-negative terms,
 *     s - g = sum_x q[x] b(rho_x),   b(rho) = phi(rho) - phi(1) - phi'(1) (rho - 1) >= 0,
 * and with a = 1/nu, t1 = 1 - a, t = 1 - a rho each term has a closed form free of cancellation:
 *     t > 0 :  b = a^2 (rho - 1)^2 H(t),   H(t) = sum_{m=0}^{K-2} (K-1-m) t1^(K-2-m) t^m
 *              (from t^K - t1^K - K t1^(K-1) (t - t1) = (t - t1)^2 H(t))
 *     t <= 0:  q b = t1^(K-1) (K a p - (1 + (K-1) a) q)          (phi(rho) = 0 there)
 * The common factor a^2 is left out (it underflows for the ratios drafts of improbable
 * tokens produce): the function returns E = nu^2 (s - g).
 *
 * The denominator c_K(P) - nu (1 - s) of Eq. (hik) equals [c_K(P) - c_K(a)] + nu (s - g), because
 * nu (1 - g) = c_K(a); and c_K(P) - c_K(a) = (a - P) S2 with
 *     S2 = sum_{j=1}^{K-1} sum_{m=0}^{j-1} (1-P)^m t1^(j-1-m) > 0,   a - P = a (1 - Q),
 * Q = nu P the joint target probability of the block.  Hence, multiplying through by nu,
 *     h_ik = E / (E + (1 - Q) S2).
 * tests/test_oracle_primitives.py checks both functions against the literal Eq. (hik) in exact
 * rational arithmetic, including block ratios of 1e30 and more.
 */
double specgbv_oracle_ot_excess(const double *lq, const double *lp, int V,
                                double log_nu, int K)
{
    if (log_nu > 690.0) log_nu = 690.0;       /* keeps nu and 1/nu finite and positive; the result no longer depends on nu there */
    const double a = exp(-log_nu);            /* 1/nu, in (0, 1) for nu > 1 */
    const double t1 = -expm1(-log_nu);        /* 1 - a */
    double E = 0.0;
    for (int x = 0; x < V; ++x) {
        const double d = lp[x] - lq[x];       /* log rho; +inf where q[x] = 0 */
        const double t = 1.0 - a * exp(d);
        if (t > 0.0) {
            double H = 0.0;                   /* sum_m (K-1-m) t1^(K-2-m) t^m */
            for (int m = 0; m <= K - 2; ++m) H += (double)(K - 1 - m) * ipow(t1, K - 2 - m) * ipow(t, m);
            const double u = expm1(d);        /* rho - 1 */
            E += exp(lq[x]) * u * u * H;
        } else {
            /* nu^2 q b = nu t1^(K-1) (K p - (nu + K - 1) q) */
            const double nu = exp(log_nu);
            E += nu * ipow(t1, K - 1) * ((double)K * exp(lp[x]) - (nu + (double)(K - 1)) * exp(lq[x]));
        }
    }
    return E;
}

/* Eq. (hik) for nu > 1 from E = nu^2 (s - g). */
double specgbv_oracle_h_sub_excess(double log_nu, double logP, double E, int K)
{
    const double t1 = -expm1(-log_nu);
    const double A = -expm1(logP);            /* 1 - P */
    double S2 = 0.0;
    for (int j = 1; j <= K - 1; ++j)
        for (int m = 0; m <= j - 1; ++m) S2 += ipow(A, m) * ipow(t1, j - 1 - m);
    const double one_minus_Q = -expm1(log_nu + logP);
    const double den = E + (one_minus_Q > 0.0 ? one_minus_Q : 0.0) * S2;
    if (!(den > 0.0)) return 1.0;             /* 0/0: limit is 1 */
    if (isinf(E)) return 1.0;
    return clamp01(E / den);
}

/* Eq. (hLk), whole block, rescaled by P_L. */
double specgbv_oracle_h_full(double log_nu, double logP, int K)
{
    const double nu = exp(log_nu);
    return clamp01(nu * (1.0 - g_K(log_nu, K)) / c_K(logP, K));
}

/* ------------------------------------------------- Algorithm 1, the scan */

static int same_block(const int32_t *a, const int32_t *b, int len)
{
    for (int j = 0; j < len; ++j)
        if (a[j] != b[j]) return 0;
    return 1;
}

/* Is the length-len block of draft k in H?  H holds (draft, length) pairs of
 * blocks that were tested and not accepted; membership is equality of the
 * token blocks. */
static int in_H(const int32_t *tokens, int L, const int *Hk, const int *Hlen,
                int nH, int k, int len)
{
    for (int e = 0; e < nH; ++e)
        if (Hlen[e] == len && same_block(tokens + (size_t)Hk[e] * L, tokens + (size_t)k * L, len))
            return 1;
    return 0;
}

/*
 * The sequential loop of Algorithm 1 for one prefix.
 *   h, eta : [K, L], entry (k, i-1) for sub-block length i
 *   tokens : [K, L]
 *   state  : [K, L] out (may be NULL): 0 = never reached, 1 = tested with
 *            its uniform, 2 = reached but skipped because the block is in H
 * Outputs tau in [0, L] and f (0-based draft index, -1 if tau = 0).
 */
void specgbv_oracle_decision_scan(const double *h, const double *eta,
                                  const int32_t *tokens, int K, int L,
                                  int32_t *tau_out, int32_t *f_out, int32_t *state)
{
    int tau = 0, f = -1, nH = 0;
    int *Hk = (int *)malloc(sizeof(int) * (size_t)K * L);
    int *Hlen = (int *)malloc(sizeof(int) * (size_t)K * L);
    if (state) memset(state, 0, sizeof(int32_t) * (size_t)K * L);

    for (int k = 0; k < K; ++k) {
        const int start = tau + 1;            /* range fixed at loop entry */
        for (int i = start; i <= L - 1; ++i) {
            if (in_H(tokens, L, Hk, Hlen, nH, k, i)) {
                if (state) state[k * L + i - 1] = 2;
                continue;                     /* no sampling for a known reject */
            }
            if (state) state[k * L + i - 1] = 1;
            if (eta[k * L + i - 1] < h[k * L + i - 1]) {
                tau = i; f = k;               /* longest accepted so far */
            } else {
                Hk[nH] = k; Hlen[nH] = i; ++nH;
            }
        }
        /* whole block */
        if (in_H(tokens, L, Hk, Hlen, nH, k, L)) {
            if (state) state[k * L + L - 1] = 2;
            continue;
        }
        if (state) state[k * L + L - 1] = 1;
        if (eta[k * L + L - 1] < h[k * L + L - 1]) {
            tau = L; f = k;
            break;
        }
        Hk[nH] = k; Hlen[nH] = L; ++nH;
    }
    free(Hk); free(Hlen);
    *tau_out = tau; *f_out = f;
}

/* ---------------------------------------------------------- final sample */

/* Inverse CDF in token-id order: the first j whose running sum exceeds u*W.
 * margin (may be NULL) = distance of u*W to the nearer end of token j's
 * interval, divided by W.  Returns -1 when W = 0. */
int32_t specgbv_oracle_sample_cdf(const double *w, int V, double u,
                                  double *W_out, double *margin)
{
    double W = 0.0;
    for (int x = 0; x < V; ++x) W += w[x];
    if (W_out) *W_out = W;
    if (!(W > 0.0)) return -1;
    const double target = u * W;
    double c = 0.0;
    int32_t last_pos = -1;
    for (int x = 0; x < V; ++x) {
        const double c_prev = c;
        c += w[x];
        if (w[x] > 0.0) last_pos = x;
        if (c > target) {
            if (margin) {
                const double lo = target - c_prev, hi = c - target;
                *margin = (lo < hi ? lo : hi) / W;
            }
            return x;
        }
    }
    if (margin) *margin = 0.0;                /* only reachable through rounding */
    return last_pos;
}

/* ------------------------------------------------------------ whole call */

/* Optional per-call intermediates (any pointer may be NULL). */
typedef struct {
    double *lse_q;      /* [B, K, L+1] log-sum-exp of target rows (z/T)      */
    double *lse_p;      /* [B, K, L]                                         */
    double *log_nu;     /* [B, K, L]   log nu_i at i-1                        */
    double *log_P;      /* [B, K, L]   log P_i at i-1                         */
    double *s;          /* [B, K, L]   OT sum of row r at r (row 0: nu = 1)   */
    double *h;          /* [B, K, L]   acceptance probability of length i    */
    double *eta;        /* [B, K, L]   uniform of that test                   */
    int32_t *state;     /* [B, K, L]   0 unreached, 1 tested, 2 skipped (H)   */
    double *res_norm;   /* [B] sum of the weights the final token is drawn from */
    double *u_final;    /* [B] uniform of the final token                     */
    double *margin;     /* [B] inverse-CDF margin of the final token          */
    int32_t *fallback;  /* [B] 1 if all residual weights were zero            */
    double *carry_log_nu;   /* [B] log of q(t^tau, y) / p(t^tau, y): the block ratio that
                             *     Algorithm 2 continues in the next iteration (0 if tau = L) */
    int32_t *modify_count;  /* [B] L - tau - 1 positions to modify next (0 if tau >= L - 1) */
} specgbv_oracle_debug;

static void verify_one(const void *target_logits, const void *draft_logits,
                       const int32_t *draft_tokens, int K, int L, int V, int b, uint32_t pid,
                       int dtype, double T, uint64_t seed, uint64_t offset,
                       int32_t *accepted_len, int32_t *accepted_draft_idx,
                       int32_t *out_tokens, const specgbv_oracle_debug *dbg)
{
    const size_t KL = (size_t)K * L;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    double *h = (double *)malloc(sizeof(double) * KL);
    double *eta = (double *)malloc(sizeof(double) * KL);
    double *log_nu = (double *)malloc(sizeof(double) * KL);
    double *log_P = (double *)malloc(sizeof(double) * KL);
    const int32_t *tokens = draft_tokens + (size_t)b * KL;

    for (int k = 0; k < K; ++k) {
        const size_t trow0 = ((size_t)b * K + k) * (size_t)(L + 1);
        const size_t drow0 = ((size_t)b * K + k) * (size_t)L;
        double lognu = 0.0, logP = 0.0;       /* nu_0 = P_0 = 1 */
        for (int r = 0; r < L; ++r) {
            load_row(target_logits, dtype, trow0 + r, V, z);
            const double lse_q = specgbv_oracle_log_softmax(z, V, T, lq);
            load_row(draft_logits, dtype, drow0 + r, V, z);
            const double lse_p = specgbv_oracle_log_softmax(z, V, T, lp);
            /* OT sum of row r with the ratio of the length-r block (r = 0: nu = 1). */
            const double s = specgbv_oracle_ot_sum(lq, lp, V, lognu, K);
            if (r >= 1) {
                /* Eq. (hik) for sub-block length i = r; for nu > 1 in the form without s - g */
                h[k * L + r - 1] = lognu > 0.0
                    ? specgbv_oracle_h_sub_excess(lognu, logP, specgbv_oracle_ot_excess(lq, lp, V, lognu, K), K)
                    : specgbv_oracle_h_sub(lognu, logP, s, K);
            }
            if (dbg) {
                if (dbg->lse_q) dbg->lse_q[trow0 + r] = lse_q;
                if (dbg->lse_p) dbg->lse_p[drow0 + r] = lse_p;
                if (dbg->s) dbg->s[drow0 + r] = s;
            }
            /* extend the block by token x^(r+1) */
            const int32_t tok = tokens[k * L + r];
            lognu += lq[tok] - lp[tok];
            logP += lp[tok];
            log_nu[k * L + r] = lognu;
            log_P[k * L + r] = logP;
        }
        /* Eq. (hLk) for the whole block */
        h[k * L + L - 1] = specgbv_oracle_h_full(lognu, logP, K);
        for (int i = 1; i <= L; ++i)
            eta[k * L + i - 1] = specgbv_oracle_uniform(seed, offset, pid,
                                                        (uint32_t)(k * L + i - 1));
    }

    int32_t tau, f;
    int32_t *state = dbg && dbg->state ? dbg->state + (size_t)b * KL : NULL;
    specgbv_oracle_decision_scan(h, eta, tokens, K, L, &tau, &f, state);

    /* final token */
    const int kf = f < 0 ? 0 : f;             /* tau = 0: row 0 of draft 0 */
    const size_t trow = ((size_t)b * K + kf) * (size_t)(L + 1) + (size_t)tau;
    load_row(target_logits, dtype, trow, V, z);
    const double lse_q = specgbv_oracle_log_softmax(z, V, T, lq);
    int fallback = 0;
    if (tau == L) {
        for (int x = 0; x < V; ++x) w[x] = exp(lq[x]);        /* bonus: y ~ q_L */
        if (dbg && dbg->lse_q) dbg->lse_q[trow] = lse_q;
    } else {
        const size_t drow = ((size_t)b * K + kf) * (size_t)L + (size_t)tau;
        load_row(draft_logits, dtype, drow, V, z);
        specgbv_oracle_log_softmax(z, V, T, lp);
        const double lognu_tau = tau == 0 ? 0.0 : log_nu[kf * L + tau - 1];
        /* Eq. (pres) with q(x^tau) cancelled */
        for (int x = 0; x < V; ++x) w[x] = ot_term(lq[x], lp[x], lognu_tau, K);
    }
    const double u = specgbv_oracle_uniform(seed, offset, pid, (uint32_t)KL);
    double W = 0.0, margin = 0.0;
    int32_t y = specgbv_oracle_sample_cdf(w, V, u, &W, &margin);
    if (y < 0) {                               /* all-zero residual: y ~ q_tau */
        fallback = 1;
        for (int x = 0; x < V; ++x) w[x] = exp(lq[x]);
        y = specgbv_oracle_sample_cdf(w, V, u, &W, &margin);
    }
    /* Algorithm 2 conditions on (t^tau, y): the block ratio extended by the final token */
    double carry = 0.0;
    if (tau < L) carry = (tau == 0 ? 0.0 : log_nu[kf * L + tau - 1]) + lq[y] - lp[y];

    accepted_len[b] = tau;
    accepted_draft_idx[b] = f;
    for (int j = 0; j <= L; ++j) {
        int32_t v = -1;
        if (j < tau) v = tokens[kf * L + j];
        else if (j == tau) v = y;
        out_tokens[(size_t)b * (L + 1) + j] = v;
    }
    if (dbg) {
        const size_t o = (size_t)b * KL;
        if (dbg->log_nu) memcpy(dbg->log_nu + o, log_nu, sizeof(double) * KL);
        if (dbg->log_P) memcpy(dbg->log_P + o, log_P, sizeof(double) * KL);
        if (dbg->h) memcpy(dbg->h + o, h, sizeof(double) * KL);
        if (dbg->eta) memcpy(dbg->eta + o, eta, sizeof(double) * KL);
        if (dbg->res_norm) dbg->res_norm[b] = W;
        if (dbg->u_final) dbg->u_final[b] = u;
        if (dbg->margin) dbg->margin[b] = margin;
        if (dbg->fallback) dbg->fallback[b] = fallback;
        if (dbg->carry_log_nu) dbg->carry_log_nu[b] = carry;
        if (dbg->modify_count) dbg->modify_count[b] = tau < L ? L - tau - 1 : 0;
    }
    free(z); free(lq); free(lp); free(w); free(h); free(eta); free(log_nu); free(log_P);
}

/*
 * Host-pointer twin of the GPU entry point.
 *   target_logits [batch, K, L+1, V], draft_logits [batch, K, L, V] (dtype:
 *   0 = float32, 1 = bfloat16 bit patterns, 2 = float64), draft_tokens [batch, K, L].
 *   Outputs accepted_len [batch], accepted_draft_idx [batch] (-1 when 0
 *   tokens are accepted), out_tokens [batch, L+1] (accepted tokens, the final
 *   token, then -1).  prefix_ids (may be NULL) gives the Philox prefix counter of each
 *   batch entry, so that a subset of a larger batch can be re-run; NULL means 0..batch-1.
 *   nthreads > 1 only distributes prefixes over threads.
 * Returns 0, or 1 for invalid arguments.
 */
int specgbv_oracle_verify(const void *target_logits, const void *draft_logits,
                          const int32_t *draft_tokens, int K, int L, int V,
                          int batch, int dtype, float temperature,
                          uint64_t rng_seed, uint64_t rng_offset,
                          int32_t *accepted_len, int32_t *accepted_draft_idx,
                          int32_t *out_tokens, const specgbv_oracle_debug *dbg,
                          const int32_t *prefix_ids, int nthreads)
{
    if (!target_logits || !draft_logits || !draft_tokens || !accepted_len ||
        !accepted_draft_idx || !out_tokens)
        return 1;
    if (K < 1 || L < 1 || V < 1 || batch < 0) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return 1;
    for (size_t j = 0; j < (size_t)batch * K * L; ++j)
        if (draft_tokens[j] < 0 || draft_tokens[j] >= V) return 1;
    const double T = (double)temperature;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int b = 0; b < batch; ++b)
        verify_one(target_logits, draft_logits, draft_tokens, K, L, V, b,
                   prefix_ids ? (uint32_t)prefix_ids[b] : (uint32_t)b, dtype, T,
                   rng_seed, rng_offset, accepted_len, accepted_draft_idx,
                   out_tokens, dbg);
    return 0;
}

int specgbv_oracle_num_procs(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* ------------------------------------------------ Algorithm 2 (next iteration) */

/*
 * Distribution modification (Algorithm 2).  After an iteration that accepted t^tau and drew
 * the final token y, the first count = L - tau - 1 positions of the next iteration use
 *     q_new(x | x^(i-1)) ~ q(t^tau, y, x^(i-1), x) (1 - min{ p(t^tau, y, x^(i-1), x) /
 *                                                        q(t^tau, y, x^(i-1), x), 1 })^K
 * instead of q.  Dividing by the joint probability of (t^tau, y, x^(i-1)) this is the same
 * per-token form as Eq. (pres),
 *     w[x] = q_r[x] max(1 - p_r[x] / (nu q_r[x]), 0)^K,   q_new = w / sum_x w,
 * with nu = [q(t^tau, y) / p(t^tau, y)] * prod_{j<r} q_j[x^(j+1)] / p_j[x^(j+1)]: the ratio
 * carried over from the previous iteration, continued along the new draft with the ORIGINAL
 * target probabilities.  If every weight is zero the row is left as q (same reading as for
 * the residual).
 *
 *   target_logits, draft_logits [batch, K, M, V]: rows r = 0..M-1 of the new drafts
 *   tokens [batch, K, M]: the new drafts' tokens (row r was sampled into tokens[r])
 *   carry_log_nu [batch], count [batch] (0..M): from the previous iteration
 *   out_logq [batch, K, M, V]: natural log of the distribution to use for row r
 *            (q_new for r < count, q otherwise; -inf where the probability is 0)
 *   norm_out [batch, K, M] (may be NULL): sum_x w of modified rows, 1 otherwise
 *   fallback_out [batch, K, M] (may be NULL): 1 where all weights were zero
 */
int specgbv_oracle_modify(const void *target_logits, const void *draft_logits,
                          const int32_t *tokens, int K, int M, int V, int batch,
                          int dtype, float temperature, const double *carry_log_nu,
                          const int32_t *count, double *out_logq, double *norm_out,
                          int32_t *fallback_out)
{
    if (!target_logits || !draft_logits || !tokens || !carry_log_nu || !count || !out_logq) return 1;
    if (K < 1 || M < 1 || V < 1 || batch < 0) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return 1;
    const double T = (double)temperature;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < batch; ++b) {
        if (count[b] < 0 || count[b] > M) { free(z); free(lq); free(lp); free(w); return 1; }
        for (int k = 0; k < K; ++k) {
            double lognu = carry_log_nu[b];
            for (int r = 0; r < M; ++r) {
                const size_t row = ((size_t)b * K + k) * (size_t)M + (size_t)r;
                load_row(target_logits, dtype, row, V, z);
                specgbv_oracle_log_softmax(z, V, T, lq);
                load_row(draft_logits, dtype, row, V, z);
                specgbv_oracle_log_softmax(z, V, T, lp);
                double *out = out_logq + row * (size_t)V;
                double W = 1.0;
                int fb = 0;
                if (r < count[b]) {
                    W = 0.0;
                    for (int x = 0; x < V; ++x) { w[x] = ot_term(lq[x], lp[x], lognu, K); W += w[x]; }
                    if (W > 0.0) {
                        for (int x = 0; x < V; ++x) out[x] = log(w[x]) - log(W);
                    } else {
                        fb = 1; W = 1.0;
                        for (int x = 0; x < V; ++x) out[x] = lq[x];
                    }
                } else {
                    for (int x = 0; x < V; ++x) out[x] = lq[x];
                }
                if (norm_out) norm_out[row] = W;
                if (fallback_out) fallback_out[row] = fb;
                const int32_t tok = tokens[row];
                if (tok < 0 || tok >= V) { free(z); free(lq); free(lp); free(w); return 1; }
                lognu += lq[tok] - lp[tok];
            }
        }
    }
    free(z); free(lq); free(lp); free(w);
    return 0;
}

/* ------------------------------------------- draft-side sampling (Algorithm 3) */

/*
 * The drafting step of Algorithm 3 ("sample x_1^L, ..., x_K^L ~ p i.i.d."): one token per row
 * from p_r = softmax(z_r / T), by the same inverse-CDF rule as the final token,
 *     y = min{ j : sum_{x<=j} p_r[x] > u },
 * with u the Philox uniform of (seed, offset, row r, slot 2^31 + position): slots from 2^31
 * upwards are never used by the verification, so the K drafts of a prefix (K rows with
 * different row indices) get independent uniforms.
 *
 *   logits [rows, V] (dtype as in specgbv_oracle_verify), out_tokens [rows],
 *   u_out, margin_out [rows] (may be NULL).  Returns 0, or 1 for invalid arguments.
 */
int specgbv_oracle_sample_rows(const void *logits, int rows, int V, int dtype,
                               float temperature, uint64_t rng_seed, uint64_t rng_offset,
                               uint32_t position, int32_t *out_tokens, double *u_out,
                               double *margin_out)
{
    if (!logits || !out_tokens || rows < 0 || V < 1) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!(temperature > 0.0f) || !isfinite(temperature) || position >= 0x80000000u) return 1;
    const double T = (double)temperature;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    for (int r = 0; r < rows; ++r) {
        load_row(logits, dtype, (size_t)r, V, z);
        specgbv_oracle_log_softmax(z, V, T, lp);
        for (int x = 0; x < V; ++x) w[x] = exp(lp[x]);
        const double u = specgbv_oracle_uniform(rng_seed, rng_offset, (uint32_t)r, 0x80000000u + position);
        double W = 0.0, margin = 0.0;
        out_tokens[r] = specgbv_oracle_sample_cdf(w, V, u, &W, &margin);
        if (u_out) u_out[r] = u;
        if (margin_out) margin_out[r] = margin;
    }
    free(z); free(lp); free(w);
    return 0;
}

/* ------------------------- pending modifications across iterations (Algorithm 3) */

/*
 * Algorithm 3 updates q in place ("q <- DistributionModification(q, p, L, t^tau, y)"), so a
 * modification that still has rows left when the next iteration ends stays in force and the
 * next one applies on top of it.  This advances ONE pending modification (carry_log_nu, count)
 * of every prefix along the tokens the iteration emitted: e_j = tokens[b, f, j] for j < tau,
 * e_tau = out_tokens[b, tau] (f = accepted draft, draft 0 when tau = 0).  With
 * q_j = softmax(rows_q[b, f, j] / T) -- the rows this modification modifies -- and p_j likewise,
 *     count > tau + 1 and tau < M:  carry += sum_{j<=tau} ln q_j[e_j] - ln p_j[e_j],  count -= tau + 1
 *     otherwise:                    count = 0   (expired)
 * because the block ratio of Algorithm 2 runs over the whole sequence (t^tau, y, x^(i-1)).
 *   rows_q [batch, K, M + bonus, V], rows_p [batch, K, M, V], tokens [batch, K, M],
 *   accepted_len, accepted_idx [batch], out_tokens [batch, M + 1].  Returns 0, or 1.
 */
int specgbv_oracle_carry_advance(const void *rows_q, const void *rows_p, const int32_t *tokens,
                                 const int32_t *accepted_len, const int32_t *accepted_idx,
                                 const int32_t *out_tokens, int K, int M, int bonus, int V,
                                 int batch, int dtype, float temperature, double *carry_log_nu,
                                 int32_t *count)
{
    if (!rows_q || !rows_p || !tokens || !accepted_len || !accepted_idx || !out_tokens || !carry_log_nu || !count)
        return 1;
    if (K < 1 || M < 1 || V < 1 || batch < 0 || (bonus != 0 && bonus != 1)) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return 1;
    const double T = (double)temperature;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < batch; ++b) {
        const int tau = accepted_len[b];
        if (tau < 0 || tau > M) { free(z); free(lq); free(lp); return 1; }
        if (tau == M || count[b] <= tau + 1) { count[b] = 0; continue; }
        const int f = accepted_idx[b] < 0 ? 0 : accepted_idx[b];
        if (f >= K) { free(z); free(lq); free(lp); return 1; }
        double c = carry_log_nu[b];
        for (int j = 0; j <= tau; ++j) {
            const int32_t e = j < tau ? tokens[((size_t)b * K + f) * M + j] : out_tokens[(size_t)b * (M + 1) + tau];
            if (e < 0 || e >= V) { free(z); free(lq); free(lp); return 1; }
            load_row(rows_q, dtype, ((size_t)b * K + f) * (size_t)(M + bonus) + (size_t)j, V, z);
            specgbv_oracle_log_softmax(z, V, T, lq);
            load_row(rows_p, dtype, ((size_t)b * K + f) * (size_t)M + (size_t)j, V, z);
            specgbv_oracle_log_softmax(z, V, T, lp);
            c += lq[e] - lp[e];
        }
        carry_log_nu[b] = c;
        count[b] -= tau + 1;
    }
    free(z); free(lq); free(lp);
    return 0;
}

/* ============================================================================
 * Comparison verifiers (paper Section 3: the methods SpecTr-GBV is measured against).
 *
 * Section 3.1, token-level speculative decoding: one draft; token x^(i) is accepted with probability
 * min{1, q(x^(i)|x^{i-1}) / p(x^(i)|x^{i-1})}; at the first rejection the replacement is drawn from
 * norm(max{q - p, 0}) of that position; if all L tokens are accepted a bonus token comes from q(.|x^L).
 *
 * Section 3.2, SpecTr with the K-SEQ rule: K i.i.d. drafts, verified position by position.  At a position the
 * candidates are the tokens of the drafts still retained (those that agree with everything accepted so far),
 * taken in draft order; a candidate x is accepted with probability min{1, q(x) / (rho p(x))}, the first accepted
 * one is emitted and the drafts that carry it stay retained; if none is accepted the replacement is drawn from
 * (q - rho min{p, q/rho}) / (1 - rho beta(rho)) and the iteration ends.  rho in [1, k] solves
 *     1 - (1 - beta(rho))^k = rho beta(rho),    beta(rho) = sum_x min{p(x), q(x)/rho}.
 * Reading taken where the text is silent: k is the number of drafts retained AT THAT POSITION (K at the first
 * one).  Only with this k is the printed residual the right one: the chance that a given token x is emitted
 * by acceptance is [1 - (1-beta)^k] / beta * min{p(x), q(x)/rho}, which must not exceed q(x) and equals
 * rho min{p, q/rho} exactly when the equation holds for the k candidates actually tested.  (Tests confirm by
 * enumeration that the emitted token is then distributed as q for every K, and is not with a fixed k = K.)
 * The distributions of a position are read from the rows of the retained draft of lowest index.
 * k = 1 gives rho = 1, i.e. Section 3.1.
 *
 * Uniforms: test of draft j at position i uses Philox slot j*L + (i-1), the final token slot K*L (the scheme
 * of the main verifier; the calls are separate, so sharing slots is harmless).
 * ========================================================================== */

/* beta(rho) = sum_x min{p[x], q[x]/rho}, plain left-to-right. */
double specgbv_oracle_kseq_beta(const double *lq, const double *lp, int V, double rho)
{
    double b = 0.0;
    for (int x = 0; x < V; ++x) {
        const double p = exp(lp[x]), qr = exp(lq[x]) / rho;
        b += p < qr ? p : qr;
    }
    return b;
}

/* f(rho) = rho beta(rho) - 1 + (1 - beta(rho))^k: non-positive at rho = 1, non-negative at rho = k, increasing. */
static double kseq_f(const double *lq, const double *lp, int V, double rho, int k)
{
    const double b = specgbv_oracle_kseq_beta(lq, lp, V, rho);
    return rho * b - 1.0 + ipow(1.0 - b, k);
}

/* The root of 1 - (1 - beta(rho))^k = rho beta(rho) in [1, k] by bisection (200 halvings at most: far below
 * one unit in the last place; the function is increasing, so the root is unique; where it vanishes on a
 * whole interval, e.g. p == q, the left end is returned). */
double specgbv_oracle_kseq_rho(const double *lq, const double *lp, int V, int k)
{
    if (k <= 1) return 1.0;
    double lo = 1.0, hi = (double)k;
    if (kseq_f(lq, lp, V, lo, k) >= 0.0) return lo;
    for (int it = 0; it < 200; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (!(mid > lo && mid < hi)) break;
        if (kseq_f(lq, lp, V, mid, k) >= 0.0) hi = mid; else lo = mid;
    }
    return hi;
}

/* Optional intermediates of the comparison verifiers (any pointer may be NULL). */
typedef struct {
    double *rho;        /* [B, L] rho used at position i (index i-1); NaN where the position was not reached  */
    double *beta;       /* [B, L] beta(rho) there                                                             */
    int32_t *retained;  /* [B, L] number of drafts retained when position i was verified (0: not reached)     */
    int32_t *lead;      /* [B, L] the retained draft of lowest index there (-1: not reached)                  */
    double *accept;     /* [B, K, L] acceptance probability of draft j's token at position i where tested    */
    double *eta;        /* [B, K, L] uniform of that test                                                     */
    int32_t *state;     /* [B, K, L] 0 not tested, 1 tested                                                   */
    double *res_norm;   /* [B] total weight the final token was drawn from (1 - rho beta, or 1 for the bonus) */
    double *u_final;    /* [B] */
    double *margin;     /* [B] */
    double *rho_all;    /* [B, K, L] eager table: rho of row r of draft j with k = number of drafts sharing   */
    double *beta_all;   /*            x_j^r (what a data-parallel implementation computes up front)          */
} specgbv_oracle_kseq_debug;

static void kseq_one(const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
                     int K, int L, int V, int b, uint32_t pid, int dtype, double T, uint64_t seed, uint64_t offset,
                     int ndrafts, int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
                     const specgbv_oracle_kseq_debug *dbg)
{
    const size_t KL = (size_t)K * L;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    int *alive = (int *)malloc(sizeof(int) * (size_t)K);
    const int32_t *tokens = draft_tokens + (size_t)b * KL;
    if (dbg) {
        for (int i = 0; i < L; ++i) {
            if (dbg->rho) dbg->rho[(size_t)b * L + i] = NAN;
            if (dbg->beta) dbg->beta[(size_t)b * L + i] = NAN;
            if (dbg->retained) dbg->retained[(size_t)b * L + i] = 0;
            if (dbg->lead) dbg->lead[(size_t)b * L + i] = -1;
        }
        for (size_t j = 0; j < KL; ++j) {
            if (dbg->accept) dbg->accept[(size_t)b * KL + j] = NAN;
            if (dbg->eta) dbg->eta[(size_t)b * KL + j] = NAN;
            if (dbg->state) dbg->state[(size_t)b * KL + j] = 0;
        }
    }
    /* eager table for parity with data-parallel implementations: every (draft, row) with its own sharing count */
    if (dbg && (dbg->rho_all || dbg->beta_all)) {
        for (int j = 0; j < ndrafts; ++j)
            for (int r = 0; r < L; ++r) {
                int k = 0;
                for (int m = 0; m < ndrafts; ++m) k += same_block(tokens + (size_t)m * L, tokens + (size_t)j * L, r);
                load_row(target_logits, dtype, ((size_t)b * K + j) * (size_t)(L + 1) + r, V, z);
                specgbv_oracle_log_softmax(z, V, T, lq);
                load_row(draft_logits, dtype, ((size_t)b * K + j) * (size_t)L + r, V, z);
                specgbv_oracle_log_softmax(z, V, T, lp);
                const double rho = specgbv_oracle_kseq_rho(lq, lp, V, k);
                if (dbg->rho_all) dbg->rho_all[(size_t)b * KL + (size_t)j * L + r] = rho;
                if (dbg->beta_all) dbg->beta_all[(size_t)b * KL + (size_t)j * L + r] = specgbv_oracle_kseq_beta(lq, lp, V, rho);
            }
    }

    int n = ndrafts, tau = 0, rejected = 0;
    for (int j = 0; j < n; ++j) alive[j] = j;
    double rho = 1.0, beta = 0.0;
    for (int i = 1; i <= L && !rejected; ++i) {
        const int r = i - 1, lead = alive[0];
        load_row(target_logits, dtype, ((size_t)b * K + lead) * (size_t)(L + 1) + r, V, z);
        specgbv_oracle_log_softmax(z, V, T, lq);
        load_row(draft_logits, dtype, ((size_t)b * K + lead) * (size_t)L + r, V, z);
        specgbv_oracle_log_softmax(z, V, T, lp);
        rho = specgbv_oracle_kseq_rho(lq, lp, V, n);
        beta = specgbv_oracle_kseq_beta(lq, lp, V, rho);
        if (dbg) {
            if (dbg->rho) dbg->rho[(size_t)b * L + r] = rho;
            if (dbg->beta) dbg->beta[(size_t)b * L + r] = beta;
            if (dbg->retained) dbg->retained[(size_t)b * L + r] = n;
            if (dbg->lead) dbg->lead[(size_t)b * L + r] = lead;
        }
        int winner = -1;
        for (int a = 0; a < n && winner < 0; ++a) {
            const int j = alive[a];
            const int32_t x = tokens[(size_t)j * L + r];
            const double ratio = exp(lq[x] - lp[x]) / rho;
            const double acc = ratio < 1.0 ? ratio : 1.0;
            const double eta = specgbv_oracle_uniform(seed, offset, pid, (uint32_t)(j * L + r));
            if (dbg) {
                if (dbg->accept) dbg->accept[(size_t)b * KL + (size_t)j * L + r] = acc;
                if (dbg->eta) dbg->eta[(size_t)b * KL + (size_t)j * L + r] = eta;
                if (dbg->state) dbg->state[(size_t)b * KL + (size_t)j * L + r] = 1;
            }
            if (eta < acc) winner = j;
        }
        if (winner < 0) { rejected = 1; break; }
        const int32_t t = tokens[(size_t)winner * L + r];
        int m = 0;
        for (int a = 0; a < n; ++a)
            if (tokens[(size_t)alive[a] * L + r] == t) alive[m++] = alive[a];
        n = m;
        tau = i;
    }
    /* final token: the residual of the position where every candidate failed, or the bonus token */
    const int lead = alive[0];
    if (rejected) {
        /* lq, lp, rho still hold that position: q - rho min{p, q/rho} = max{q - rho p, 0} */
        for (int x = 0; x < V; ++x) {
            const double q = exp(lq[x]), p = exp(lp[x]);
            const double m = p < q / rho ? p : q / rho;
            w[x] = q - rho * m;
            if (w[x] < 0.0) w[x] = 0.0;
        }
    } else {
        load_row(target_logits, dtype, ((size_t)b * K + lead) * (size_t)(L + 1) + L, V, z);
        specgbv_oracle_log_softmax(z, V, T, lq);
        for (int x = 0; x < V; ++x) w[x] = exp(lq[x]);
    }
    const double u = specgbv_oracle_uniform(seed, offset, pid, (uint32_t)KL);
    double W = 0.0, margin = 0.0;
    int32_t y = specgbv_oracle_sample_cdf(w, V, u, &W, &margin);
    if (y < 0) {                                 /* only through rounding (a rejection needs 1 - rho beta > 0) */
        for (int x = 0; x < V; ++x) w[x] = exp(lq[x]);
        y = specgbv_oracle_sample_cdf(w, V, u, &W, &margin);
    }
    accepted_len[b] = tau;
    if (accepted_draft_idx) accepted_draft_idx[b] = tau > 0 ? lead : -1;
    for (int j = 0; j <= L; ++j) {
        int32_t v = -1;
        if (j < tau) v = tokens[(size_t)lead * L + j];
        else if (j == tau) v = y;
        out_tokens[(size_t)b * (L + 1) + j] = v;
    }
    if (dbg) {
        if (dbg->res_norm) dbg->res_norm[b] = W;
        if (dbg->u_final) dbg->u_final[b] = u;
        if (dbg->margin) dbg->margin[b] = margin;
    }
    free(z); free(lq); free(lp); free(w); free(alive);
}

/*
 * SpecTr K-SEQ verification (Section 3.2) on the inputs of specgbv_oracle_verify, using the first `ndrafts`
 * of the K drafts (ndrafts = K: SpecTr; ndrafts = 1: rho = 1, i.e. token-level speculative decoding).
 * accepted_draft_idx (may be NULL) receives the retained draft of lowest index, -1 when nothing was accepted.
 * Returns 0, or 1 for invalid arguments.
 */
int specgbv_oracle_verify_kseq(const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
                               int K, int L, int V, int batch, int dtype, float temperature,
                               uint64_t rng_seed, uint64_t rng_offset, int ndrafts,
                               int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
                               const specgbv_oracle_kseq_debug *dbg, const int32_t *prefix_ids, int nthreads)
{
    if (!target_logits || !draft_logits || !draft_tokens || !accepted_len || !out_tokens) return 1;
    if (K < 1 || L < 1 || V < 1 || batch < 0 || ndrafts < 1 || ndrafts > K) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return 1;
    for (size_t j = 0; j < (size_t)batch * K * L; ++j)
        if (draft_tokens[j] < 0 || draft_tokens[j] >= V) return 1;
    const double T = (double)temperature;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int b = 0; b < batch; ++b)
        kseq_one(target_logits, draft_logits, draft_tokens, K, L, V, b,
                 prefix_ids ? (uint32_t)prefix_ids[b] : (uint32_t)b, dtype, T, rng_seed, rng_offset, ndrafts,
                 accepted_len, accepted_draft_idx, out_tokens, dbg);
    return 0;
}

/*
 * Token-level speculative decoding (Section 3.1) written out from its own definition, on draft 0 of the same
 * inputs: accept x^(i) with probability min{1, q/p}, residual norm(max{q - p, 0}), bonus token after L
 * acceptances.  Same uniforms as specgbv_oracle_verify_kseq with ndrafts = 1 (slot i-1, final slot K*L), so the
 * two must agree token for token: that is one of the pins of the K-SEQ code.
 */
int specgbv_oracle_verify_token_sd(const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
                                   int K, int L, int V, int batch, int dtype, float temperature,
                                   uint64_t rng_seed, uint64_t rng_offset, int32_t *accepted_len, int32_t *out_tokens)
{
    if (!target_logits || !draft_logits || !draft_tokens || !accepted_len || !out_tokens) return 1;
    if (K < 1 || L < 1 || V < 1 || batch < 0) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    if (!(temperature > 0.0f) || !isfinite(temperature)) return 1;
    const double T = (double)temperature;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    double *w = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < batch; ++b) {
        const int32_t *tok = draft_tokens + (size_t)b * K * L;     /* draft 0 */
        int tau = 0, rejected = 0;
        for (int i = 1; i <= L; ++i) {
            load_row(target_logits, dtype, ((size_t)b * K) * (size_t)(L + 1) + (i - 1), V, z);
            specgbv_oracle_log_softmax(z, V, T, lq);
            load_row(draft_logits, dtype, ((size_t)b * K) * (size_t)L + (i - 1), V, z);
            specgbv_oracle_log_softmax(z, V, T, lp);
            const int32_t x = tok[i - 1];
            if (x < 0 || x >= V) { free(z); free(lq); free(lp); free(w); return 1; }
            const double ratio = exp(lq[x] - lp[x]);
            const double alpha = ratio < 1.0 ? ratio : 1.0;
            if (specgbv_oracle_uniform(rng_seed, rng_offset, (uint32_t)b, (uint32_t)(i - 1)) < alpha) { tau = i; continue; }
            for (int v = 0; v < V; ++v) {
                const double d = exp(lq[v]) - exp(lp[v]);
                w[v] = d > 0.0 ? d : 0.0;
            }
            rejected = 1;
            break;
        }
        if (!rejected) {
            load_row(target_logits, dtype, ((size_t)b * K) * (size_t)(L + 1) + L, V, z);
            specgbv_oracle_log_softmax(z, V, T, lq);
            for (int v = 0; v < V; ++v) w[v] = exp(lq[v]);
        }
        const double u = specgbv_oracle_uniform(rng_seed, rng_offset, (uint32_t)b, (uint32_t)(K * L));
        int32_t y = specgbv_oracle_sample_cdf(w, V, u, NULL, NULL);
        if (y < 0) {
            for (int v = 0; v < V; ++v) w[v] = exp(lq[v]);
            y = specgbv_oracle_sample_cdf(w, V, u, NULL, NULL);
        }
        accepted_len[b] = tau;
        for (int j = 0; j <= L; ++j) out_tokens[(size_t)b * (L + 1) + j] = j < tau ? tok[j] : (j == tau ? y : -1);
    }
    free(z); free(lq); free(lp); free(w);
    return 0;
}
