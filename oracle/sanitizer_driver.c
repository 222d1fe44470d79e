/*
 * sanitizer_driver.c -- runs the oracle's entry points on small seeded inputs and prints what they return.
 *
 * TEST INFRASTRUCTURE ONLY.  tests/test_oracle_sanitizers.py compiles this file together with specgbv_oracle.c
 * under -fsanitize=address,undefined (any report aborts the run) and compares the printed results with those the
 * ordinary build of the oracle gives, through its Python wrapper, on the same inputs; the inputs come from the
 * 64-bit linear congruential generator below, which the test reproduces.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    double *lse_q, *lse_p, *log_nu, *log_P, *s, *h, *eta; int32_t *state;
    double *res_norm, *u_final, *margin; int32_t *fallback; double *carry_log_nu; int32_t *modify_count;
} dbg_t;
typedef struct {
    double *rho, *beta; int32_t *retained, *lead; double *accept, *eta; int32_t *state;
    double *res_norm, *u_final, *margin, *rho_all, *beta_all;
} kdbg_t;

int specgbv_oracle_verify(const void *, const void *, const int32_t *, int, int, int, int, int, float, uint64_t, uint64_t,
                          int32_t *, int32_t *, int32_t *, const dbg_t *, const int32_t *, int);
int specgbv_oracle_verify_kseq(const void *, const void *, const int32_t *, int, int, int, int, int, float, uint64_t, uint64_t,
                               int, int32_t *, int32_t *, int32_t *, const kdbg_t *, const int32_t *, int);
int specgbv_oracle_verify_token_sd(const void *, const void *, const int32_t *, int, int, int, int, int, float, uint64_t,
                                   uint64_t, int32_t *, int32_t *);
int specgbv_oracle_modify(const void *, const void *, const int32_t *, int, int, int, int, int, float, const double *,
                          const int32_t *, double *, double *, int32_t *);
int specgbv_oracle_sample_rows(const void *, int, int, int, float, uint64_t, uint64_t, uint32_t, int32_t *, double *, double *);
int specgbv_oracle_carry_advance(const void *, const void *, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                                 int, int, int, int, int, int, float, double *, int32_t *);

static uint64_t lcg_state;
static double lcg_unit(void)               /* in [0, 1): top 53 bits of a 64-bit LCG */
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(lcg_state >> 11) * (1.0 / 9007199254740992.0);
}

int main(void)
{
    enum { B = 5, K = 3, L = 4, V = 37 };
    const size_t nt = (size_t)B * K * (L + 1) * V, nd = (size_t)B * K * L * V, n = (size_t)B * K * L;
    float *t = malloc(sizeof(float) * nt), *d = malloc(sizeof(float) * nd);
    int32_t *tok = malloc(sizeof(int32_t) * n);
    lcg_state = 12345;
    for (size_t i = 0; i < nt; ++i) t[i] = (float)(6.0 * lcg_unit() - 3.0);
    for (size_t i = 0; i < nd; ++i) d[i] = (float)(6.0 * lcg_unit() - 3.0);
    for (size_t i = 0; i < n; ++i) tok[i] = (int32_t)(lcg_unit() * V);
    t[7] = -INFINITY;                          /* a masked target entry */
    int32_t acc[B], idx[B], out[B * (L + 1)];
    double h[B * K * L], s[B * K * L], lognu[B * K * L], carry[B];
    int32_t state[B * K * L], mcount[B];
    dbg_t dbg = {0};
    dbg.h = h; dbg.s = s; dbg.log_nu = lognu; dbg.state = state; dbg.carry_log_nu = carry; dbg.modify_count = mcount;
    for (int off = 0; off < 3; ++off) {
        if (specgbv_oracle_verify(t, d, tok, K, L, V, B, 0, 0.9f, 77, (uint64_t)off, acc, idx, out, &dbg, NULL, 2)) return 2;
        printf("verify %d:", off);
        for (int b = 0; b < B; ++b) printf(" %d %d", acc[b], idx[b]);
        for (int j = 0; j < B * (L + 1); ++j) printf(" %d", out[j]);
        double hs = 0.0; for (size_t j = 0; j < n; ++j) hs += h[j];
        printf(" %.12e\n", hs);
    }
    /* Algorithm 2 and the advance of its ratio, fed by the last verification */
    double *logq = malloc(sizeof(double) * nd), norm[B * K * L];
    int32_t fb[B * K * L];
    if (specgbv_oracle_modify(t, d, tok, K, L, V, B, 0, 0.9f, carry, mcount, logq, norm, fb)) return 3;
    double ns = 0.0; for (size_t j = 0; j < n; ++j) ns += norm[j];
    printf("modify: %.12e\n", ns);
    if (specgbv_oracle_carry_advance(t, d, tok, acc, idx, out, K, L, 1, V, B, 0, 0.9f, carry, mcount)) return 4;
    printf("advance:"); for (int b = 0; b < B; ++b) printf(" %.12e %d", carry[b], mcount[b]); printf("\n");
    /* comparison verifiers */
    double rho[B * L], rall[B * K * L];
    kdbg_t kd = {0};
    kd.rho = rho; kd.rho_all = rall;
    for (int ndr = 1; ndr <= K; ++ndr) {
        if (specgbv_oracle_verify_kseq(t, d, tok, K, L, V, B, 0, 0.9f, 78, 1, ndr, acc, idx, out, &kd, NULL, 1)) return 5;
        printf("kseq %d:", ndr);
        for (int b = 0; b < B; ++b) printf(" %d %d", acc[b], idx[b]);
        for (int j = 0; j < B * (L + 1); ++j) printf(" %d", out[j]);
        double rs = 0.0; for (int b = 0; b < B; ++b) for (int k = 0; k < ndr; ++k) for (int r = 0; r < L; ++r) rs += rall[((size_t)b * K + k) * L + r];
        printf(" %.12e\n", rs);
    }
    if (specgbv_oracle_verify_token_sd(t, d, tok, K, L, V, B, 0, 0.9f, 78, 1, acc, out)) return 6;
    printf("sd:"); for (int b = 0; b < B; ++b) printf(" %d", acc[b]); for (int j = 0; j < B * (L + 1); ++j) printf(" %d", out[j]); printf("\n");
    /* drafting step */
    int32_t drawn[B * K]; double u[B * K], mg[B * K];
    if (specgbv_oracle_sample_rows(d, B * K, V, 0, 0.9f, 5, 6, 2, drawn, u, mg)) return 7;
    printf("sample:"); for (int j = 0; j < B * K; ++j) printf(" %d", drawn[j]); printf("\n");
    free(t); free(d); free(tok); free(logq);
    return 0;
}
