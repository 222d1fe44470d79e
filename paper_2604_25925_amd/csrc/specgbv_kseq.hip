// Comparison verifier: SpecTr's K-SEQ rule (paper Section 3.2), and with one draft token-level speculative
// decoding (Section 3.1), on the inputs of the main verification.
//
// At a position the candidates are the tokens of the drafts still retained (those that agree with everything
// accepted so far), taken in draft order; candidate x is accepted with probability min{1, q(x) / (rho p(x))}, and
// if none is accepted the replacement is drawn from (q - rho min{p, q/rho}) / (1 - rho beta(rho)) = norm(max{q - rho p, 0}).
// rho in [1, k] solves 1 - (1 - beta(rho))^k = rho beta(rho), beta(rho) = sum_x min{p(x), q(x)/rho}, with k the
// number of drafts retained at that position.
//
// Which drafts are retained when a position is reached depends only on the tokens: they are the drafts that share
// the accepted block, and the accepted block is always some draft's prefix.  So the root can be found up front
// for every (draft, row), with k = the number of drafts sharing that draft's first r tokens -- all row pairs in
// parallel, no dependence on the random decisions.  That is what k_kseq_rows does:
//     rho beta(rho) = 1 - S(rho),   S(rho) = sum_x max{q - rho p, 0} = sum_x q max(1 - rho p/q, 0)
// is the K = 1 vocabulary sum of the main verifier at block ratio 1/rho, so one sweep over the row pair gives S and
// its slope (-sum_{rho p < q} p), and a safeguarded Newton iteration on f(rho) = (1 - beta)^k - S finds the root in
// a handful of sweeps.  The sequential part (which candidate wins at each position) is then a scalar scan per
// prefix inside the final-token kernel, and the replacement token is that kernel's K = 1 residual draw.
#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kKseqThreads = 512;
// the sweeps of a workgroup read the same row pair again and again: ordinary loads, not the streaming ones
// (2 - 7 % faster: part of a sweep is then served by the cache levels in front of HBM)
constexpr bool kKseqKeep = true;

// G(rho) = sum_x min{rho p, q} = rho beta(rho), S(rho) = sum_x max{q - rho p, 0} = 1 - G, and rho * sum_{rho p < q} p.
// G and S are summed separately and normalised by their own total, so that each keeps its leading digits where it is
// small (G where the models hardly overlap, S where they nearly coincide) whatever the accuracy of the row's normaliser.
struct KseqSums { double G, S, Dr; };

// One sweep over the row pair at scale rho.  C1 = log2 Z_p - log2 Z_q; weights relative to 2^shift_q.
template <typename T, bool VEC>
__device__ __forceinline__ KseqSums kseq_sweep(const T *rq, const T *rp, int V, float c, float shift_q, double C1,
                                               double rho, double *sh_d)
{
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    const RatioConst rc(C1 - log2(rho));                  // rho p / q = 2^(c (z_p - z_q) - C2)
    const float kappa = -rc.neg_kappa;
    // summed as min{rho p, q} (not as max{q - rho p, 0} = q - min): where the two models hardly overlap the sum is
    // tiny and the equation for rho is decided by its leading digits
    float G = 0.0f, S = 0.0f, Dr = 0.0f;
    for_each_pair<T, VEC, kKseqThreads, kKseqKeep>(rq, rp, V, [&](int, const float (&zq)[N], const float (&zp)[N]) {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const float r = exp2_fast(fmaf(zp[j] - zq[j], c, -rc.C2_hi)) * kappa;        // rho p / q
            const float e = exp2_fast(fmaf(zq[j], c, -shift_q));
            const bool open = r < 1.0f;                                                   // rho p < q
            G = fmaf(e, open ? r : 1.0f, G);
            S = fmaf(e, open ? 1.0f - r : 0.0f, S);
            Dr += open ? e * r : 0.0f;
        }
    });
    KseqSums out;
    out.G = block_sum(static_cast<double>(G), sh_d);
    out.S = block_sum(static_cast<double>(S), sh_d);
    out.Dr = block_sum(static_cast<double>(Dr), sh_d);
    const double tot = out.G + out.S;                      // = sum_x q in the sums' own units
    if (tot > 0.0) { out.G /= tot; out.S /= tot; out.Dr /= tot; }
    return out;
}

// grid batch * ndrafts * L: workgroup (b, k, r) takes row pair r of draft k of prefix b: its statistics, the number
// n of drafts (among the first ndrafts) that share the draft's first r tokens, and the root rho for k = n.
template <typename T, bool VEC>
__global__ void __launch_bounds__(kKseqThreads)
k_kseq_rows(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens, int K, int L,
            int V, int ndrafts, float c, double c_rel, RowStat *__restrict__ stats, double *__restrict__ rho_out,
            double *__restrict__ beta_out, int32_t *__restrict__ final_counter)
{
    __shared__ double sh_d[kKseqThreads / kWave];
    __shared__ float sh_f[kKseqThreads / kWave];
    __shared__ int sh_n;
    const int r = static_cast<int>(blockIdx.x % L);
    const long long bkd = blockIdx.x / L;
    const int k = static_cast<int>(bkd % ndrafts);
    const long long b = bkd / ndrafts;
    const long long bk = b * K + k, pair = bk * L + r;
    const int tid = threadIdx.x;
    if (tid == 0) {
        sh_n = 0;
        if (k == 0 && r == 0) final_counter[b] = 0;       // arrival counter of the final-token kernel
    }
    __syncthreads();
    if (tid < ndrafts) {
        bool same = true;
        for (int j = 0; j < r; ++j) same = same && tokens[(b * K + tid) * L + j] == tokens[bk * L + j];
        if (same) atomicAdd(&sh_n, 1);
    }
    const T *rq = target + (bk * (L + 1) + r) * static_cast<long long>(V);
    const T *rp = draft + pair * static_cast<long long>(V);
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    RunningSum aq, ap;
    for_each_pair<T, VEC, kKseqThreads, kKseqKeep>(rq, rp, V, [&](int, const float (&zq)[N], const float (&zp)[N]) {
        aq.add(zq, c);
        ap.add(zp, c);
    });
    const float Mq = block_max(aq.m2, sh_f);
    const double Zq = block_sum(aq.Z > 0.0f ? static_cast<double>(aq.Z) * exp2(static_cast<double>(aq.m2) - static_cast<double>(Mq)) : 0.0, sh_d);
    const float Mp = block_max(ap.m2, sh_f);
    const double Zp = block_sum(ap.Z > 0.0f ? static_cast<double>(ap.Z) * exp2(static_cast<double>(ap.m2) - static_cast<double>(Mp)) : 0.0, sh_d);
    const double lse2_q = static_cast<double>(Mq) + log2(Zq), lse2_p = static_cast<double>(Mp) + log2(Zp);
    if (tid == 0) {
        int tok = tokens[pair];
        tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
        RowStat st;
        st.lse2_q = lse2_q; st.lse2_p = lse2_p;
        st.tok2_q = token_scaled(static_cast<double>(Elem<T>::scalar(rq + tok)) * static_cast<double>(c), lse2_q, c_rel);
        st.tok2_p = token_scaled(static_cast<double>(Elem<T>::scalar(rp + tok)) * static_cast<double>(c), lse2_p, c_rel);
        stats[pair] = st;
    }
    const int n = sh_n;                                    // (the block sums above contain the barriers that publish it)
    const float shift_q = rintf(static_cast<float>(lse2_q));
    const double C1 = lse2_p - lse2_q;

    // f(rho) = G(rho) - 1 + (1 - beta)^n, beta = G / rho: non-positive at 1, non-negative at n, increasing.  It is
    // evaluated as G + expm1(n log1p(-beta)), which keeps its leading digits when G is tiny.  Newton from the left end,
    // kept inside the bracket by bisection, until the step is below 2e-7 rho (or f is below the noise of the float32
    // sums); every quantity is workgroup-uniform.
    double rho = 1.0, lo = 1.0, hi = static_cast<double>(n), beta = 0.0;
    for (int it = 0;; ++it) {
        const KseqSums sm = kseq_sweep<T, VEC>(rq, rp, V, c, shift_q, C1, rho, sh_d);
        beta = sm.G / rho;
        if (n <= 1) break;                                 // one candidate: rho = 1 (Section 3.1)
        const double b1 = beta < 1.0 ? beta : 1.0;
        // (1 - beta)^n - S, or G + [(1 - beta)^n - 1]: the same number, each form exact where the other cancels
        const double f = b1 > 0.5 ? exp(static_cast<double>(n) * log1p(-b1 < -1.0 ? -1.0 : -b1)) - sm.S
                                  : sm.G + expm1(static_cast<double>(n) * log1p(-b1));
        if (fabs(f) <= 1.0e-7 * fmin(sm.G, sm.S) || hi - lo <= 2.0e-7 * rho || it >= 40) break;   // (rho, beta): the pair just evaluated
        if (f >= 0.0) hi = rho; else lo = rho;
        const double D = sm.Dr / rho;                      // d(rho beta)/d rho = mass of p where rho p < q
        const double pw1 = b1 < 1.0 ? exp(static_cast<double>(n - 1) * log1p(-b1)) : 0.0;
        const double fp = D - static_cast<double>(n) * pw1 * (D - beta) / rho;
        double nxt = fp > 0.0 ? rho - f / fp : 0.5 * (lo + hi);
        if (!(nxt > lo && nxt < hi)) nxt = 0.5 * (lo + hi);
        if (fabs(nxt - rho) <= 2.0e-7 * rho && it > 0) break;
        rho = nxt;
    }
    if (tid == 0) { rho_out[pair] = rho; beta_out[pair] = beta; }
}

template <typename T>
hipError_t launch_kseq_typed(const Problem &p, int ndrafts)
{
    const T *target = static_cast<const T *>(p.target);
    const T *draft = static_cast<const T *>(p.draft);
    const bool vec = (p.V % Elem<T>::kPerVec) == 0 && (reinterpret_cast<uintptr_t>(p.target) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(p.draft) % 16 == 0);
    const dim3 grid(static_cast<unsigned>(static_cast<long long>(p.batch) * ndrafts * p.L));
    RowStat *stats = reinterpret_cast<RowStat *>(p.ws + p.lay.stats);
    double *rho = reinterpret_cast<double *>(p.ws + p.lay.s);
    double *beta = reinterpret_cast<double *>(p.ws + p.lay.excess);
    int32_t *counter = reinterpret_cast<int32_t *>(p.ws + p.lay.counter);
    if (vec)
        hipLaunchKernelGGL((k_kseq_rows<T, true>), grid, dim3(kKseqThreads), 0, p.stream, target, draft, p.tokens, p.K, p.L,
                           p.V, ndrafts, p.c, p.c_rel, stats, rho, beta, counter);
    else
        hipLaunchKernelGGL((k_kseq_rows<T, false>), grid, dim3(kKseqThreads), 0, p.stream, target, draft, p.tokens, p.K, p.L,
                           p.V, ndrafts, p.c, p.c_rel, stats, rho, beta, counter);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_kseq_rows(const Problem &p, int ndrafts)
{
    return p.dtype == 1 ? launch_kseq_typed<uint16_t>(p, ndrafts) : launch_kseq_typed<float>(p, ndrafts);
}

}  // namespace specgbv
