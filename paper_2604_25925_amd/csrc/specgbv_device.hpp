// Device-side helpers shared by the SpecTr-GBV kernels (gfx950, wave64).
//
// Arithmetic conventions used by every kernel:
//   * logits are scaled to base-2 exponents with one float constant
//       c = float(log2(e) / temperature)
//     and the same float is used (widened) on the float64 scalar side, so all
//     GPU-side quantities are mutually consistent;
//   * vocabulary-wide sums are accumulated per thread in float32 and combined
//     across threads in float64;
//   * O(batch*K*L) scalars (block ratios, acceptance probabilities) are float64.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specgbv {

constexpr int kWave = 64;

// ---------------------------------------------------------------- workspace

// Per (prefix, draft, row) statistics, all in base-2 logarithms.
struct RowStat {
    double lse2_q;   // log2 sum_x 2^(c z_q[x])
    double lse2_p;   // log2 sum_x 2^(c z_p[x])
    double tok2_q;   // c * z_q[token of this row]
    double tok2_p;   // c * z_p[token of this row]
};

// Pending distribution modifications (Algorithm 2 applied on the fly, possibly several on top of
// each other: Algorithm 3 updates q in place).  Level l turns the row's distribution q^(l) into
//   q^(l+1)[x] = q^(l)[x] t_l[x]^K / N_l,   t_l[x] = max(1 - p[x] / (mu_l q^(l)[x]), 0),   q^(0) = q,
// for the first count_l rows of every draft.  Per (level, prefix, draft, row), in base-2 logarithms:
constexpr int kMaxPend = 16;     // levels applied on the fly at most
constexpr double kExcessPending = -2.0;   // in the array of E = nu^2 (s - g): the row's sum is on its way, in parts (chain schedule)
constexpr int kMaxDrafts = 64;   // K at most (one lane of a wave per draft where the drafts of a prefix are compared)
struct PendRow {
    double log2mu;   // block ratio mu_l in front of this row (carried ratio continued along the drafted tokens with q^(l))
    double log2N;    // log2 of N_l = sum_x q^(l)[x] t_l[x]^K (0 when the level does not modify the row)
    double tokadj;   // K log2 t_l[token of this row]: log2 q^(l+1)[token] = log2 q^(l)[token] + tokadj - log2N (0 when not modified)
    int32_t flag;    // 1: the level modifies the row; 0: row beyond its count, or N_l = 0 (the row stays q^(l))
    int32_t pad;
};

// Constants of the levels that modify one row, in order (workgroup-uniform; kept in LDS):
// p[x] / (mu_l q^(l)[x]) = 2^(c (z_p - z_q) - C_hi[l]) kappa_l / T_l[x] with T_l = prod_{m<l} t_m^K.
struct PendTable {
    int n;
    float C_hi[kMaxPend];
    float neg_kappa[kMaxPend];
};

// What the final-token kernels need to know about one prefix.
struct Selection {
    long long target_row;   // row index into target_logits (in rows of V elements)
    long long draft_row;    // row index into draft_logits, or -1 for the bonus row
    double C2;              // log2 of nu * Z_p / Z_q: the ratio p/(nu q) is 2^(c (z_p - z_q) - C2)
    double lse2_q;          // log2 normaliser of the target row (0 for the bonus row)
    float shift_q;          // reference exponent for target-row weights (unused for the bonus row)
    int tau;
    int npend;              // levels of pending modifications that modify the row (C2 and lse2_q then refer to the modified row)
    float C2_adj;           // added to C2 where it serves the sweep's ratio: minus c_rel log2 nu (see ratio_const)
    double lse2_pq;         // log2 Z_p - log2 Z_q of the unmodified row pair (0 for the bonus row)
    double Cl[kMaxPend];    // per such level: log2 of mu_l Z_p / Z_q minus the log2 N of the levels before it
};

// Partial sums of one residual segment, relative to 2^m2.
struct SegPartial {
    double sum_w;    // sum of residual weights
    double sum_q;    // sum of plain target weights (used if every residual weight is zero)
    float m2;        // reference exponent of both sums
    float pad;
};

// The drafted token's scaled logit as RowStat keeps it: c z[token], adjusted so that tok2 - lse2 is the token's
// log2 probability at the caller's temperature.  The kernels scale logits with the float c, which differs from
// log2(e) / T by the relative amount c_rel (at most 6e-8 in magnitude); a token far below the bulk of its row
// (hundreds of base-2 units at a low temperature) would carry that relative error into the block ratio in
// full.  To first order the log-probability of such a token is proportional to the scale, so it is rescaled;
// for tokens near the bulk the adjustment is far below the arithmetic's own error.
// A token the model gives probability zero (logit -inf) keeps its -inf.
__device__ __forceinline__ double token_scaled(double tok2, double lse2, double c_rel)
{
    const double d = tok2 - lse2;
    return (d - d == 0.0) ? tok2 + c_rel * d : tok2;      // (d - d is 0 for finite d and not a number otherwise)
}

// ------------------------------------------------------------------- loads

struct alignas(16) U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerVec = 4;       // elements per 16-byte load
    __device__ static __forceinline__ void unpack(const U4 &v, float (&o)[4]) {
        o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y);
        o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
    }
    __device__ static __forceinline__ float scalar(const float *p) { return *p; }
    // one element as loaded (no arithmetic on it, so that nothing has to wait for the load) and its value
    __device__ static __forceinline__ uint32_t bits(const float *p) { return *reinterpret_cast<const uint32_t *>(p); }
    __device__ static __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }
};
template <> struct Elem<uint16_t> {
    static constexpr int kPerVec = 8;
    __device__ static __forceinline__ void unpack(const U4 &v, float (&o)[8]) {
        o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
        o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
    }
    __device__ static __forceinline__ float scalar(const uint16_t *p) {
        return __uint_as_float(static_cast<uint32_t>(*p) << 16);
    }
    __device__ static __forceinline__ uint32_t bits(const uint16_t *p) { return *p; }
    __device__ static __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b << 16); }
};

__device__ __forceinline__ U4 load16(const void *p) {
    return *reinterpret_cast<const U4 *>(p);
}

// The same with the non-temporal hint, for logits that are streamed once per kernel: they are not kept in the
// cache levels in front of HBM, which on this chip raises the streaming rate noticeably (measured on the chain
// kernel: float32 rows 69 % -> 76 % of the HBM peak).
__device__ __forceinline__ U4 load16_stream(const void *p) {
    typedef unsigned int V4 __attribute__((ext_vector_type(4)));
    const V4 v = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(p));
    return U4{v.x, v.y, v.z, v.w};
}

// ------------------------------------------------------------------- math

// v_exp_f32: 2^x, about 1 ulp, flushes results below 2^-126.
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// max(1 - r, 0) for r >= 0, as one clamped subtract.
__device__ __forceinline__ float one_minus_clamped(float r) {
    return __builtin_amdgcn_fmed3f(1.0f - r, 0.0f, 1.0f);
}

// The ratio p[x] / (nu q[x]) = 2^(c (z_p - z_q) - C2) with a float64 constant C2 that can be
// large while the exponent itself is small for the entries that matter.  C2 is split into
// a float part used inside the exponent and a factor kappa = 2^-(C2 - float(C2)) applied in
// the following "1 - ratio" (as one fused multiply-add), so the rounding of C2 to float
// costs neither accuracy nor an instruction.
struct RatioConst {
    float C2_hi;
    float neg_kappa;
    __device__ __forceinline__ explicit RatioConst(double C2) {
        C2_hi = static_cast<float>(C2);
        const double kappa = exp2(static_cast<double>(C2_hi) - C2);
        neg_kappa = (kappa > 0.5 && kappa < 2.0) ? -static_cast<float>(kappa) : -1.0f;   // non-finite C2
    }
    // max(1 - p/(nu q), 0) for logit difference d = z_p - z_q
    __device__ __forceinline__ float one_minus_ratio(float d, float c) const {
        const float r = __builtin_amdgcn_exp2f(fmaf(d, c, -C2_hi));
        return __builtin_amdgcn_fmed3f(fmaf(r, neg_kappa, 1.0f), 0.0f, 1.0f);
    }
};

// C2 for the sweeps' ratio p[x] / (nu q[x]) = 2^(c (z_p - z_q) - C2), C2 = log2 Z_p - log2 Z_q + log2 nu, with the part
// of the rounding of c that a constant can carry.  The float c differs from log2(e) / T by the relative amount
// c_rel, which puts c_rel (c (z_p - z_q) - (E_p[c z] - E_q[c z])) into the exponent (the normalisers, summed with the
// same c, move with it).  For the entries whose ratio is of order one - the only ones whose factor 1 - ratio is
// sensitive - c (z_p - z_q) is C2 itself up to a few units, i.e. the error is c_rel (log2 nu + H_p - H_q) with the
// two rows' entropies in bits: a block ratio of 2^-28 (a long block of improbable tokens) shifts every such ratio by
// 1e-6, and the K-th power of a factor 0.2 by 1e-5.  The log2 nu part is taken out here; the entropies are not known.
__device__ __forceinline__ double ratio_const(double lse2_p, double lse2_q, double log2nu, double c_rel)
{
    return (lse2_p - lse2_q) + log2nu * (1.0 - c_rel);
}

// 2^x in float64 (0 below x = -1000, infinity above x = 1000) by a degree-12 polynomial on [-1/2, 1/2] and an exponent shift
// (relative error about 1e-15; far less code than the general library routine, which matters
// in kernels whose run time is mostly instruction fetch, and few registers, which matters where
// the register file is full of data).
__device__ __forceinline__ double exp2_small(double x)
{
    if (!(x > -1000.0)) return 0.0;
    if (x > 1000.0) return INFINITY;
    const double n = rint(x);
    const double f = (x - n) * 0.693147180559945309417;      // |f| <= 0.3466
    double p = 1.0 / 479001600.0;
    p = fma(p, f, 1.0 / 39916800.0);
    p = fma(p, f, 1.0 / 3628800.0);
    p = fma(p, f, 1.0 / 362880.0);
    p = fma(p, f, 1.0 / 40320.0);
    p = fma(p, f, 1.0 / 5040.0);
    p = fma(p, f, 1.0 / 720.0);
    p = fma(p, f, 1.0 / 120.0);
    p = fma(p, f, 1.0 / 24.0);
    p = fma(p, f, 1.0 / 6.0);
    p = fma(p, f, 0.5);
    p = fma(p, f, 1.0);
    p = fma(p, f, 1.0);
    return ldexp(p, static_cast<int>(n));
}

// max(1 - kappa r / tK, 0) for the second ratio of a row under a pending modification: r / tK is
// formed with the hardware reciprocal (1 ulp); tK = 0, an overflowing quotient and 0/0-like cases
// (the entry's weight q tK is then zero or negligible) give 0.
__device__ __forceinline__ float pend_second_factor(float r, float tK, float neg_kappa) {
    const float q2 = r * __builtin_amdgcn_rcpf(tK);
    const float t2 = __builtin_amdgcn_fmed3f(fmaf(q2, neg_kappa, 1.0f), 0.0f, 1.0f);
    return (tK > 0.0f && q2 < 4.0f) ? t2 : 0.0f;       // kappa < 2: beyond 4 the factor is 0 anyway
}

// t^K for a wave-uniform integer K >= 1 (square and multiply).
__device__ __forceinline__ float powi_uniform(float t, int K) {
    float acc = (K & 1) ? t : 1.0f;
    float base = t;
    for (int k = K >> 1; k; k >>= 1) {
        base *= base;
        if (k & 1) acc *= base;
    }
    return acc;
}

__device__ __forceinline__ double powi_uniform(double t, int K) {
    double acc = (K & 1) ? t : 1.0;
    double base = t;
    for (int k = K >> 1; k; k >>= 1) {
        base *= base;
        if (k & 1) acc *= base;
    }
    return acc;
}

// t[j] <- t[j]^K for a wave-uniform integer K >= 1, all N entries together: the entries' multiply chains are
// independent, so one uniform loop over the bits of K serves them all (a loop per entry would serialise
// N short dependent chains behind N sets of branches).
template <int N>
__device__ __forceinline__ void pow_array(float (&t)[N], int K) {
    if (K == 1) return;
    if (K == 2 || K == 4 || K == 8 || K == 16) {
#pragma unroll
        for (int j = 0; j < N; ++j) t[j] *= t[j];
        if (K >= 4) {
#pragma unroll
            for (int j = 0; j < N; ++j) t[j] *= t[j];
        }
        if (K >= 8) {
#pragma unroll
            for (int j = 0; j < N; ++j) t[j] *= t[j];
        }
        if (K >= 16) {
#pragma unroll
            for (int j = 0; j < N; ++j) t[j] *= t[j];
        }
        return;
    }
    float base[N];
#pragma unroll
    for (int j = 0; j < N; ++j) { base[j] = t[j]; t[j] = (K & 1) ? t[j] : 1.0f; }
    for (int k = K >> 1; k; k >>= 1) {
#pragma unroll
        for (int j = 0; j < N; ++j) base[j] *= base[j];
        if (k & 1) {
#pragma unroll
            for (int j = 0; j < N; ++j) t[j] *= base[j];
        }
    }
}

// Weights of N entries of a (target, draft) row pair relative to 2^shift_q:
//   wq[j] = 2^(c z_q[j] - shift_q)                      (plain target weight)
//   w[j]  = wq[j] max(1 - p[j] / (nu q[j]), 0)^K        (the terms of Eq. (hik) / Eq. (pres)), nu in rc.
template <int N>
__device__ __forceinline__ void ot_weights(const float (&zq)[N], const float (&zp)[N], float c, float shift_q,
                                           const RatioConst &rc, int K, float (&wq)[N], float (&w)[N]) {
    float t[N];
#pragma unroll
    for (int j = 0; j < N; ++j) t[j] = rc.one_minus_ratio(zp[j] - zq[j], c);
    pow_array(t, K);
#pragma unroll
    for (int j = 0; j < N; ++j) { wq[j] = exp2_fast(fmaf(zq[j], c, -shift_q)); w[j] = wq[j] * t[j]; }
}

// The same for a row under pending modifications (tab: the levels that modify it, at least one): with T = prod_l t_l^K,
//   wq[j] = 2^(c z_q[j] - shift_q) T[j]                 (plain weight of the modified row, up to 1 / prod N_l)
//   w[j]  = wq[j] max(1 - p[j] / (nu q'[j]), 0)^K       with nu / prod N_l in rc: every level's ratio is the first
//                                                       kind of exponential divided by the running product T.
template <int N>
__device__ __forceinline__ void pending_weights(const float (&zq)[N], const float (&zp)[N], float c, float shift_q,
                                                const PendTable &tab, const RatioConst &rc, int K, float (&wq)[N],
                                                float (&w)[N]) {
    float T[N], d[N];
    {                                                 // level 0 (tab.n >= 1): T = 1, no quotient
        const float C_hi = tab.C_hi[0], neg_kappa = tab.neg_kappa[0];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            d[j] = zp[j] - zq[j];
            T[j] = __builtin_amdgcn_fmed3f(fmaf(exp2_fast(fmaf(d[j], c, -C_hi)), neg_kappa, 1.0f), 0.0f, 1.0f);
        }
        pow_array(T, K);
    }
    for (int l = 1; l < tab.n; ++l) {                 // uniform
        const float C_hi = tab.C_hi[l], neg_kappa = tab.neg_kappa[l];
        float t[N];
#pragma unroll
        for (int j = 0; j < N; ++j) t[j] = pend_second_factor(exp2_fast(fmaf(d[j], c, -C_hi)), T[j], neg_kappa);
        pow_array(t, K);
#pragma unroll
        for (int j = 0; j < N; ++j) T[j] *= t[j];
    }
    float t[N];
#pragma unroll
    for (int j = 0; j < N; ++j) t[j] = pend_second_factor(exp2_fast(fmaf(d[j], c, -rc.C2_hi)), T[j], rc.neg_kappa);
    pow_array(t, K);
#pragma unroll
    for (int j = 0; j < N; ++j) { wq[j] = exp2_fast(fmaf(zq[j], c, -shift_q)) * T[j]; w[j] = wq[j] * t[j]; }
}

// ---- Eq. (hik) for a block ratio nu > 1 without the difference s - g.
//
// s = E_q phi(rho) and g = phi(1) = phi(E_q rho) with phi(rho) = max(1 - rho/nu, 0)^K convex and rho = p[x]/q[x]
// of mean one under q, so s - g = sum_x q[x] b(rho_x) with the non-negative convexity remainder
// b(rho) = phi(rho) - phi(1) - phi'(1) (rho - 1).  With a = 1/nu, t1 = 1 - a, t = 1 - a rho:
//     t > 0 :  b = a^2 (rho - 1)^2 H(t),   H(t) = sum_{m=0}^{K-2} (K-1-m) t1^(K-2-m) t^m
//     t <= 0:  q b = t1^(K-1) (K a p - (1 + (K-1) a) q)
// The kernels sum E = nu^2 (s - g), i.e. the terms without the factor a^2 (which underflows for the ratios that
// drafts of improbable tokens produce); the decision then takes h = E / (E + (1 - Q) S2).  When s and g agree to
// several digits (peaked rows, large nu) this is the only way to get h right in float32 arithmetic, so the sum
// kernels evaluate it for exactly those rows (excess_wanted) on top of s.
struct ExcessConst {
    float c;
    float shift_q, shift_p;    // reference exponents: q[x] ~ 2^(c z_q - shift_q), p[x] ~ 2^(c z_p - shift_p) in the same units
    float C1_hi, kappa;        // rho = kappa 2^(c (z_p - z_q) - C1_hi), C1 = log2 Z_p - log2 Z_q
    float a, t1, nu;           // 1/nu (not below 1e-30), 1 - a, nu (not above 1e30)
    float Kk, nuK1, lead;      // K kappa_p; nu + K - 1; nu t1^(K-1)
    int K;
    double scale;              // 2^(shift_q - log2 Z_q): the sum of the terms times this is E
};

__device__ __forceinline__ ExcessConst make_excess_const(double lse2_q, double lse2_p, double log2nu, int K, float c)
{
    ExcessConst ec;
    ec.c = c; ec.K = K;
    ec.shift_q = rintf(static_cast<float>(lse2_q));
    const double C1 = lse2_p - lse2_q;
    const RatioConst rc(C1);
    ec.C1_hi = rc.C2_hi; ec.kappa = -rc.neg_kappa;
    const double sp = static_cast<double>(ec.shift_q) + C1;
    ec.shift_p = static_cast<float>(sp);
    const double kp = exp2_small(static_cast<double>(ec.shift_p) - sp);      // what rounding shift_p leaves out
    double a = exp2_small(-log2nu);
    if (!(a > 1.0e-30)) a = 1.0e-30;
    const double nu = 1.0 / a, t1 = 1.0 - a;
    ec.a = static_cast<float>(a); ec.t1 = static_cast<float>(t1); ec.nu = static_cast<float>(nu);
    ec.Kk = static_cast<float>(static_cast<double>(K) * ((kp > 0.5 && kp < 2.0) ? kp : 1.0));
    ec.nuK1 = static_cast<float>(nu + static_cast<double>(K - 1));
    ec.lead = static_cast<float>(nu * powi_uniform(t1, K - 1));
    ec.scale = exp2_small(static_cast<double>(ec.shift_q) - lse2_q);
    return ec;
}

// Sum over N entries of the terms of E.
template <int N>
__device__ __forceinline__ float excess_terms(const float (&zq)[N], const float (&zp)[N], const ExcessConst &ec)
{
    float rho[N], eq[N], t[N], H[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        rho[j] = ec.kappa * exp2_fast(fmaf(zp[j] - zq[j], ec.c, -ec.C1_hi));     // +inf where q[x] = 0
        eq[j] = exp2_fast(fmaf(zq[j], ec.c, -ec.shift_q));
        t[j] = fmaf(-ec.a, rho[j], 1.0f);
        H[j] = ec.K >= 2 ? 1.0f : 0.0f;                                          // coefficient of t^(K-2)
    }
    float pw = 1.0f;                                                             // t1^(K-2-m)
    for (int m = ec.K - 3; m >= 0; --m) {                                        // uniform; Horner in t
        pw *= ec.t1;
        const float cm = static_cast<float>(ec.K - 1 - m) * pw;
#pragma unroll
        for (int j = 0; j < N; ++j) H[j] = fmaf(H[j], t[j], cm);
    }
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const float u = rho[j] - 1.0f;
        const float open = (eq[j] * u) * u * H[j];
        const float ep = exp2_fast(fmaf(zp[j], ec.c, -ec.shift_p));
        const float shut = ec.lead * fmaf(ec.Kk, ep, -ec.nuK1 * eq[j]);
        acc += (t[j] > 0.0f) ? open : fmaxf(shut, 0.0f);                         // entries masked in both models: 0
    }
    return acc;
}

// Largest s / (s - g) at which the plain sum s still serves.  The sum of a row that a few entries dominate carries the
// float32 error of those entries unaveraged: 1e-7 for each of its two exponentials and K times that, plus the
// roundings of the multiplications, through the power (3e-7 observed at K = 4 on a 526-entry row, 1.3e-6 at K = 9 on
// a row with 83 % of the sum in one entry).  Taken as 2e-7 + 1.3e-7 K relative, times this factor it stays at half the
// 1e-5 the acceptance probability is held to: 15 at K = 1, 6.9 at K = 4, 4 at K = 8.
__device__ __forceinline__ float cancel_factor(int K) { return fminf(16.0f, 38.5f / (1.54f + static_cast<float>(K))); }

// Do s and g agree so closely (block ratio above one) that nu (s - g) needs the sum E?
// (float32 throughout: the threshold need not be sharp, and float64 constants in a kernel whose registers hold a
// whole row pair end up in scratch memory)
__device__ __forceinline__ bool excess_wanted(float l, float sf, int K)
{
    if (!(l > 0.0f)) return false;
    const float t1 = 1.0f - exp2_fast(-l);
    const float g = powi_uniform(t1, K);
    return (sf - g) * cancel_factor(K) < sf;
}

// Does the acceptance probability of a row whose s and g nearly cancel (excess_wanted) need the sum E at all?
// With h = E / (E + D), D = (1 - Q) S2 / nu (the decision kernel's form of Eq. (hik) for a block ratio above one), a
// relative error on E = nu (s - g) reaches h reduced by the factor 1 - h = D / (D + E): a block that is accepted
// almost surely does not care how well s - g is known.  The test of excess_wanted, sharpened by that factor, which
// is itself taken at the low end of what the plain s allows for s - g (three times the sum's error below it, 1e-6 s at
// K = 1; not above 0: needed).
// log2P: log2 of the joint draft probability of the block's tokens.
__device__ __forceinline__ bool excess_needed(double log2nu, double log2P, double s, int K)
{
    if (K == 1) return false;                   // S2 is empty: h = 1 whatever E is
    const double inv_nu = exp2_small(-log2nu), P = exp2_small(log2P);
    const double t1 = 1.0 - inv_nu, A = 1.0 - P;
    double g = 1.0;
    for (int j = 0; j < K; ++j) g *= t1;
    double U = 1.0, S2 = 0.0, pw = 1.0;
    for (int j = 1; j <= K - 1; ++j) { S2 += U; pw *= t1; U = fma(A, U, pw); }
    const double one_Q = fmax(1.0 - exp2_small(log2nu + log2P), 0.0);
    const double D = inv_nu * one_Q * S2;
    const double f = static_cast<double>(cancel_factor(K));
    const double x = (s - g) - (16.0e-6 / f) * s;
    if (!(x > 0.0)) return true;
    return x * f * (D + x / inv_nu) < s * D;
}

// Entry l of a PendTable from the float64 constant C (same split as RatioConst).
__device__ __forceinline__ void pend_table_set(PendTable &tab, int l, double C) {
    const RatioConst rc(C);
    tab.C_hi[l] = rc.C2_hi;
    tab.neg_kappa[l] = rc.neg_kappa;
}

// The levels (0 .. nlev-1, arrays level-major with n_rows entries each) that modify row `pair`, as a table of
// constants; base = log2 Z_p - log2 Z_q of the row.  Returns the sum of their log2 N.
__device__ __forceinline__ double pend_build_table(const PendRow *pend, long long n_rows, int nlev, long long pair, double base,
                                   PendTable &tab)
{
    double sumN = 0.0;
    int n = 0;
    for (int l = 0; l < nlev; ++l) {
        const PendRow pr = pend[static_cast<long long>(l) * n_rows + pair];
        if (pr.flag) {
            pend_table_set(tab, n, base + pr.log2mu - sumN);
            ++n;
            sumN += pr.log2N;
        }
    }
    tab.n = n;
    return sumN;
}

// log2 q^(nlev)[token] - log2 q[token] of row `pair`: what levels 0 .. nlev-1 do to the drafted token's probability.
__device__ __forceinline__ double pend_token_adjust(const PendRow *pend, long long n_rows, int nlev, long long pair)
{
    double a = 0.0;
    for (int l = 0; l < nlev; ++l) a += pend[l * n_rows + pair].tokadj - pend[l * n_rows + pair].log2N;
    return a;
}

// ------------------------------------------------------- row-pair streaming

// f(first entry index, z_q[N], z_p[N]) for the entries of a (target, draft) row pair in the unit range [lo, hi),
// N = 8 or 4 entries of one 16-byte vector (VEC; a unit is a vector) or 1 (a unit is an entry); the workgroup's
// THREADS threads stride over the range, each keeping the loads of two vectors of either row in flight.
// KEEP: the rows are read again soon (by the same workgroup), so they are loaded without the non-temporal hint.
template <typename T, bool VEC, int THREADS, bool KEEP = false, typename F>
__device__ __forceinline__ void for_each_pair_range(const T *rq, const T *rp, int lo, int hi, F f)
{
    constexpr int PV = Elem<T>::kPerVec;
    auto ld = [](const T *p) { return KEEP ? load16(p) : load16_stream(p); };
    if constexpr (VEC) {
        int v = lo + static_cast<int>(threadIdx.x);
        for (; v + THREADS < hi; v += 2 * THREADS) {             // four loads in flight per thread
            const U4 q0 = ld(rq + static_cast<long long>(v) * PV), p0 = ld(rp + static_cast<long long>(v) * PV);
            const U4 q1 = ld(rq + static_cast<long long>(v + THREADS) * PV);
            const U4 p1 = ld(rp + static_cast<long long>(v + THREADS) * PV);
            float zq[PV], zp[PV];
            Elem<T>::unpack(q0, zq); Elem<T>::unpack(p0, zp); f(v * PV, zq, zp);
            Elem<T>::unpack(q1, zq); Elem<T>::unpack(p1, zp); f((v + THREADS) * PV, zq, zp);
        }
        if (v < hi) {
            float zq[PV], zp[PV];
            Elem<T>::unpack(ld(rq + static_cast<long long>(v) * PV), zq);
            Elem<T>::unpack(ld(rp + static_cast<long long>(v) * PV), zp);
            f(v * PV, zq, zp);
        }
    } else {
        for (int x = lo + static_cast<int>(threadIdx.x); x < hi; x += THREADS) {
            const float zq[1] = {Elem<T>::scalar(rq + x)}, zp[1] = {Elem<T>::scalar(rp + x)};
            f(x, zq, zp);
        }
    }
}

// The whole row pair.
template <typename T, bool VEC, int THREADS, bool KEEP = false, typename F>
__device__ __forceinline__ void for_each_pair(const T *rq, const T *rp, int V, F f)
{
    for_each_pair_range<T, VEC, THREADS, KEEP>(rq, rp, 0, VEC ? V / Elem<T>::kPerVec : V, f);
}


// ------------------------------------------------------------ running sum

// Per-thread running sum of 2^(c z - m2) with a running reference exponent m2 (updated once
// per 16-byte vector; the partial sum is rescaled when the reference moves).
struct RunningSum {
    float m2 = -3.0e38f;          // finite, so that -inf logits give 2^(-inf) = 0, not NaN
    float Z = 0.0f;
    template <int N>
    __device__ __forceinline__ void add(const float (&z)[N], float c) {
        float vm = z[0];
#pragma unroll
        for (int j = 1; j < N; ++j) vm = fmaxf(vm, z[j]);
        const float n2 = fmaxf(m2, vm * c);
        float a = 0.0f;
#pragma unroll
        for (int j = 0; j < N; ++j) a += exp2_fast(fmaf(z[j], c, -n2));
        Z = fmaf(Z, exp2_fast(m2 - n2), a);
        m2 = n2;
    }
};

// The drafted token is left out of a row's float32 sums: `here` says that the vector z holds it, as entry `elem`, and
// its weight becomes 2^(-inf) = 0.  Its weight is added in float64 where the row's partial sums meet (with_token).
// A row whose mass sits on its drafted token (probability 0.9999 and beyond: low temperatures) then keeps the mass of
// all the OTHER entries to float32 relative accuracy, and 1 - P, 1 - Q and the factor's distance from one in
// Eq. (hik) are made of exactly that; summed together with a weight near one it would be known to 6e-8 absolute.
template <int N>
__device__ __forceinline__ void leave_out(float (&z)[N], bool here, int elem)
{
    if (here) {
        asm volatile("");                       // (keeps this a branch that all other waves skip)
#pragma unroll
        for (int j = 0; j < N; ++j) z[j] = j == elem ? -__builtin_inff() : z[j];
    }
}

// The drafted token's index for leave_out, fetched by a vector load from an address the compiler cannot see is
// uniform: it then queues with the row's loads.  (A scalar load is waited for where its result is first needed,
// and everything derived from a loop-invariant index is needed before the loop: one memory latency in front of the
// first row load, on kernels that consist of two or three such latencies when the batch is small.)
__device__ __forceinline__ int token_index_queued(const int32_t *tokens, long long at)
{
    int zero = 0;
    asm volatile("" : "+v"(zero));
    return tokens[at + zero];
}
// ... and clamped to the vocabulary where it is used; opaque, so that the use stays behind the loads issued before it.
__device__ __forceinline__ int token_index_used(int raw, int V)
{
    asm volatile("" : "+v"(raw));
    return raw < 0 ? 0 : (raw >= V ? V - 1 : raw);
}

// Z 2^M + 2^t as Z' 2^ref: a sum of weights relative to 2^M (M finite) and one more entry with scaled logit t
// (t = -inf: a masked entry, weight 0).
struct RefSum { double ref, Z; };
__device__ __forceinline__ RefSum with_token(double M, double Z, double t)
{
    RefSum r;
    r.ref = fmax(M, t);
    r.Z = (Z > 0.0 ? Z * exp2(M - r.ref) : 0.0) + exp2(t - r.ref);
    return r;
}

// The drafted token's term q[x] max(1 - p[x]/(nu q[x]), 0)^K of its own row's Eq. (hik) sum, in float64 from the
// row's statistics: log2q = log2 q[x], log2r = log2 of p[x]/(nu q[x]).  The sweeps form 1 - ratio per entry from a
// float32 exponential, 6e-8 absolute at ratios near one; where the token's ratio is within kTokenTermBelow of one the
// kernels replace the sweep's value of this one term (a row whose mass sits on its drafted token, behind a block
// ratio near one, has little else in the sum; at K = 1 the sum is then off by 1e-5 - 1e-4 otherwise).
constexpr float kTokenTermBelow = 0.0625f;
struct TokenTerm {
    float zq, zp;            // the token's two logits as the sweep sees them
    double log2q, log2r;
};
__device__ __forceinline__ double token_term(double log2q, double log2r, int K)
{
    const double t = fmax(1.0 - exp2_small(log2r), 0.0);
    return exp2_small(log2q) * powi_uniform(t, K);
}

// Integral reference exponent of a group of entries whose largest logit is m (partial sums taken relative to
// integral references rescale exactly).  A group without a finite entry (m = -3e38 or -inf: every entry
// masked) gets the finite reference -3e38, against which all its weights are 2^(-inf) = 0.
__device__ __forceinline__ float integral_reference(float m, float c) { return ceilf(fmaxf(m * c, -3.0e38f)); }

// Exponent shift from one integral reference to a larger one, bounded so that the conversion to int is defined;
// below 2^-4000 every partial sum is 0 in float64 anyway.
__device__ __forceinline__ int reference_shift(float from, float to) { return static_cast<int>(fmaxf(from - to, -4000.0f)); }

// ------------------------------------------------------------- reductions

// Wave-wide reductions with data-parallel-primitive moves instead of LDS permutes: shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then the two row broadcasts (lane 15 -> next row of
// each half, lane 31 -> upper half).  The sequence is an inclusive scan in lane order; lane 63
// ends up with the reduction over all 64 lanes.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move(double v) {
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(b), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(b >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned>(lo));
}

// Inclusive prefix sum over the wave in lane order (lanes without a source add +0.0).
__device__ __forceinline__ double wave_inclusive_sum(double v) {
    v += dpp_move<0x111, 0xf>(v);       // row_shr:1
    v += dpp_move<0x112, 0xf>(v);       // row_shr:2
    v += dpp_move<0x114, 0xf>(v);       // row_shr:4
    v += dpp_move<0x118, 0xf>(v);       // row_shr:8
    v += dpp_move<0x142, 0xa>(v);       // row_bcast:15 into rows 1 and 3
    v += dpp_move<0x143, 0xc>(v);       // row_bcast:31 into rows 2 and 3
    return v;
}

// Sum over the wave; every lane gets the result.
__device__ __forceinline__ double wave_sum(double v) {
    const long long b = __double_as_longlong(wave_inclusive_sum(v));
    const unsigned lo = __builtin_amdgcn_readlane(static_cast<int>(b), 63);
    const unsigned hi = __builtin_amdgcn_readlane(static_cast<int>(b >> 32), 63);
    return __longlong_as_double(static_cast<long long>((static_cast<unsigned long long>(hi) << 32) | lo));
}

// Sum over the wave in float32 (DPP adds fused into the moves); every lane gets the result.
__device__ __forceinline__ float wave_sum_f32(float v) {
#define SPECGBV_ADD_STEP(CTRL, ROW_MASK) \
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false))
    SPECGBV_ADD_STEP(0x111, 0xf);
    SPECGBV_ADD_STEP(0x112, 0xf);
    SPECGBV_ADD_STEP(0x114, 0xf);
    SPECGBV_ADD_STEP(0x118, 0xf);
    SPECGBV_ADD_STEP(0x142, 0xa);
    SPECGBV_ADD_STEP(0x143, 0xc);
#undef SPECGBV_ADD_STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Maximum over the wave; every lane gets the result.  Lanes without a source keep their own value.
__device__ __forceinline__ float wave_max(float v) {
#define SPECGBV_MAX_STEP(CTRL, ROW_MASK)                                                                   \
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, \
                                                            ROW_MASK, 0xf, false)))
    SPECGBV_MAX_STEP(0x111, 0xf);
    SPECGBV_MAX_STEP(0x112, 0xf);
    SPECGBV_MAX_STEP(0x114, 0xf);
    SPECGBV_MAX_STEP(0x118, 0xf);
    SPECGBV_MAX_STEP(0x142, 0xa);
    SPECGBV_MAX_STEP(0x143, 0xc);
#undef SPECGBV_MAX_STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Sum over the workgroup; every thread gets the result.  `scratch` holds at least
// (blockDim.x / 64) doubles of LDS; safe to call repeatedly with the same scratch.
__device__ __forceinline__ double block_sum(double v, double *scratch) {
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    const int nw = (blockDim.x + kWave - 1) / kWave;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) scratch[wid] = v;
    __syncthreads();
    double r = 0.0;
    for (int w = 0; w < nw; ++w) r += scratch[w];
    return r;
}

// log2 of the block ratio in front of row i of the draft whose rows start at row0: the sum over rows j < i of
// log2 q'_j[token] - log2 p_j[token], with q' the target row as levels 0 .. nlev-1 of the pending modifications
// leave it (pend may be null when nlev = 0).  All threads of the workgroup take part (every term is one
// independent load; a single thread walking them would pay each load's latency in turn).
__device__ __forceinline__ double pend_block_ratio(const RowStat *stats, const PendRow *pend, long long n_rows, int nlev,
                                                   long long row0, int i, double *scratch) {
    double v = 0.0;
    const int per = nlev + 1;
    for (int t = threadIdx.x; t < i * per; t += blockDim.x) {
        const int j = t / per, l = t % per;
        if (l == nlev) {
            const RowStat a = stats[row0 + j];
            v += (a.tok2_q - a.lse2_q) - (a.tok2_p - a.lse2_p);
        } else {
            const PendRow pr = pend[l * n_rows + row0 + j];
            v += pr.tokadj - pr.log2N;
        }
    }
    return block_sum(v, scratch);
}

__device__ __forceinline__ float block_max(float v, float *scratch) {
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    const int nw = (blockDim.x + kWave - 1) / kWave;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) scratch[wid] = v;
    __syncthreads();
    float r = scratch[0];
    for (int w = 1; w < nw; ++w) r = fmaxf(r, scratch[w]);
    return r;
}

// ------------------------------------------------------------------ Philox

// Philox4x32-10 (Salmon et al., SC'11); returns output word 0.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c0;
}

// Uniform in [0,1) with 24 random bits for (seed, offset, prefix, slot).
__device__ __forceinline__ double philox_uniform(uint64_t seed, uint64_t offset, uint32_t prefix,
                                                 uint32_t slot) {
    const uint32_t w = philox4x32_10_word0(static_cast<uint32_t>(offset), static_cast<uint32_t>(offset >> 32),
                                           prefix, slot, static_cast<uint32_t>(seed),
                                           static_cast<uint32_t>(seed >> 32));
    return static_cast<double>(w >> 8) * (1.0 / 16777216.0);
}

}  // namespace specgbv
