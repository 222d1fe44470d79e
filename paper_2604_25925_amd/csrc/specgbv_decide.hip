// Decision scan of Algorithm 1 and the final-token draw, in one kernel.
//
// k_final runs on a grid of (segment groups, prefixes); a workgroup has four waves and each
// wave owns four consecutive 512-entry vocabulary segments of the row the final token is drawn from.
//   1. decision  : every workgroup of a prefix rebuilds the prefix's decision (it is a few
//                  microseconds of scalar work and saves a kernel boundary): nu_i, P_i, the
//                  acceptance table (Eq. (hik) for i < L, Eq. (hLk) for i = L, both divided
//                  through by P_i so that no joint block probability is ever formed), the
//                  Philox uniforms, then the sequential loop with the set H of rejected
//                  blocks on the first wave.  The first workgroup of the prefix writes the
//                  outputs and intermediates.
//   2. partials  : per segment, the sum of the weights the final token is drawn from --
//                  Eq. (pres) with q(x^tau) cancelled, w[x] = q[x] max(1 - p[x]/(nu q[x]), 0)^K,
//                  or q[x] for the bonus token.
//   3. locate    : the workgroup that finishes last for its prefix (a counter in the
//                  workspace, zeroed by the streaming kernel that runs before) does the
//                  inverse-CDF search: the first token id whose running weight exceeds
//                  u * total (segment by a workgroup-wide scan of the partial sums, entry by
//                  a wave scan inside that segment).
#include <cstdlib>

#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kDecideThreads = 256;
constexpr int kSegPerWave = 4;               // residual segments per wave of the final-token kernel

// ---------------------------------------------------------------- k_decide

// (1 - (1-P)^K) / P = sum_{j<K} (1-P)^j: chance that one of K i.i.d. drafts equals a block of
// draft probability P, over P.  The geometric sum has no cancellation for tiny P (it tends to K)
// and costs K - 1 fused multiply-adds instead of a log1p and an expm1.
__device__ double c_K(double P, int K)
{
    if (!(P > 0.0)) return static_cast<double>(K);
    if (P >= 1.0) return 1.0;
    const double a = 1.0 - P;
    double c = 1.0;
    for (int j = 1; j < K; ++j) c = fma(c, a, 1.0);
    return c;
}

// max(1 - 1/nu, 0)^K from 1/nu.
__device__ double g_K(double inv_nu, int K)
{
    const double t = 1.0 - inv_nu;
    return t > 0.0 ? powi_uniform(t, K) : 0.0;
}

// Bitwise OR over the 64 lanes of the wave with data-parallel-primitive moves (row shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then the two row broadcasts), result read from lane 63.
__device__ __forceinline__ unsigned wave_or32(unsigned v)
{
    v |= static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x111, 0xf, 0xf, false));   // row_shr:1
    v |= static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x112, 0xf, 0xf, false));   // row_shr:2
    v |= static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x114, 0xf, 0xf, false));   // row_shr:4
    v |= static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x118, 0xf, 0xf, false));   // row_shr:8
    v |= static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x142, 0xa, 0xf, false));   // row_bcast:15
    v |= static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x143, 0xc, 0xf, false));   // row_bcast:31
    return static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}

__device__ __forceinline__ unsigned long long wave_or64(unsigned long long v)
{
    return (static_cast<unsigned long long>(wave_or32(static_cast<unsigned>(v >> 32))) << 32) |
           wave_or32(static_cast<unsigned>(v));
}

__device__ __forceinline__ unsigned long long uniform_u64(unsigned long long v)
{
    return (static_cast<unsigned long long>(__builtin_amdgcn_readfirstlane(static_cast<unsigned>(v >> 32))) << 32) |
           static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<unsigned>(v)));
}

__device__ double clamp01(double h)
{
    if (!(h > 0.0)) return 0.0;
    return h < 1.0 ? h : 1.0;
}

// A double of lane `src` (wave-uniform) in every lane.
__device__ __forceinline__ double lane_value(double v, int src)
{
    const long long bits = __double_as_longlong(v);
    const unsigned lo = __builtin_amdgcn_readlane(static_cast<int>(bits), src);
    const unsigned hi = __builtin_amdgcn_readlane(static_cast<int>(bits >> 32), src);
    return __longlong_as_double(static_cast<long long>((static_cast<unsigned long long>(hi) << 32) | lo));
}

struct DecideIO {
    const int32_t *tokens;
    const RowStat *stats;
    const PendRow *pend;        // rows under pending modifications [nlev][n_rows], or null
    long long n_rows;           // batch * K * L
    int nlev;
    const double *s_arr;
    const double *e_arr;        // nu^2 (s - g) of Eq. (hik) where the sum kernels took it without cancellation, else negative
    const double *e_part;       // chain schedule: the parts of the rows marked kExcessPending
    const double *s_part;       // s_parts > 1: the sums arrive as s_parts partial sums per row ([n_rows][kPendParts])
    double *s_store;            //              and the complete ones are stored here by the writing workgroup
    int s_parts;
    int e_parts;                // > 0: an entry kExcessPending of e_arr stands for the sum of the row's first e_parts parts
    int e_coop;                 // != 0 (two-pass schedule): nobody has looked yet whether a row needs E; the
                                // workgroups of the prefix find out and sum it together (e_part_rw: parts, each -1 until there)
    double *e_part_rw;
    int e_polls;                // looks a workgroup takes at a part another one sums before it sums the part itself
    double *log_nu_out, *log_P_out, *h_out, *eta_out;
    int32_t *state_out;
    int32_t *accepted_len, *accepted_draft_idx, *out_tokens;
    double c_rel;               // relative rounding error of the float scale c (token_scaled)
    int kseq_ndrafts;           // > 0: comparison verifier (K-SEQ rule) on the first kseq_ndrafts drafts; s_arr then holds
                                // rho and e_arr beta(rho) of every row pair
    int32_t *kseq_pos;          // [2][batch * L] drafts retained at each position reached, and the lowest of them
};

// Decision of prefix b by the whole workgroup (kDecideThreads threads); the result is left in
// *sel_out (shared memory) and is visible to every thread on return.  Only a workgroup with
// write = true stores outputs and intermediates.  *u_final_out (shared memory) receives the uniform
// of the final token (Philox slot K*L), drawn here so that the generator is instantiated once.
// excess_sums(tq, tp, lq, lp, ex): called by all threads (behind a barrier) when io.e_coop is set and some entry of
// ex has been marked kExcessPending by the acceptance table's loop below; it replaces every marked entry by the
// row's E = nu^2 (s - g) and ends with a barrier.
template <typename Hook>
__device__ __forceinline__ void decide_prefix(const DecideIO &io, int b, int K, int L, uint64_t seed, uint64_t offset,
                                              bool write, double *lds, Selection *sel_out, double *u_final_out,
                                              PendTable *tab_out, Hook excess_sums)
{
    const int32_t *__restrict__ tokens = io.tokens;
    const RowStat *__restrict__ stats = io.stats;
    const double *__restrict__ s_arr = io.s_arr;
    const int KL = K * L;
    double *l2nu = lds;                                     // [K*L] log2 nu_i
    double *tq = lds + KL;                                  // [K*L] log2 q_r[token of row r]
    double *tp = lds + 2 * KL;                              // [K*L] log2 p_r[token of row r]
    double *lq = lds + 3 * KL;                              // [K*L] log2 normaliser of target row r
    double *lp = lds + 4 * KL;                              // [K*L] log2 normaliser of draft row r
    double *ex = lds + 5 * KL;                              // [K*L] nu^2 (s - g) where it was summed without cancellation, else < 0
    unsigned long long *acc_bits = reinterpret_cast<unsigned long long *>(lds + 6 * KL);   // [K] bit i: eta_{k,i} < h_{k,i}
    int *tok = reinterpret_cast<int *>(acc_bits + K);       // [K*L]
    unsigned char *cpl = reinterpret_cast<unsigned char *>(tok + KL);   // [K*K] common prefix lengths (at most L <= 62)
    const int tid = threadIdx.x;
    const long long base = static_cast<long long>(b) * KL;
    constexpr double kLn2 = 0.693147180559945309417;

    for (int idx = tid; idx < K; idx += kDecideThreads) acc_bits[idx] = 0ull;
    for (int idx = tid; idx < KL; idx += kDecideThreads) {
        const RowStat st = stats[base + idx];
        tq[idx] = st.tok2_q - st.lse2_q;
        if (io.pend) tq[idx] += pend_token_adjust(io.pend, io.n_rows, io.nlev, base + idx);   // log2 q'[token]
        tp[idx] = st.tok2_p - st.lse2_p;
        lq[idx] = st.lse2_q; lp[idx] = st.lse2_p;
        tok[idx] = tokens[base + idx];
        // the Eq. (hik) sum this thread needs for entry idx of the table below, loaded alongside the statistics
        // (one memory latency instead of two); parked where the entry's log2 nu goes afterwards
        const int k = idx / L, i = idx % L + 1;
        double s = 0.0, e = -1.0;
        if (i < L) {
            if (io.s_parts > 1) {                           // in part order: the same bits in every workgroup
                for (int q = 0; q < io.s_parts; ++q) s += io.s_part[(base + k * L + i) * kPendParts + q];
                if (write) io.s_store[base + k * L + i] = s;
            } else {
                s = s_arr[base + k * L + i];
                e = io.e_arr[base + k * L + i];
                if (io.e_parts > 0 && e == kExcessPending) {    // (in part order: the same bits in every workgroup)
                    e = 0.0;
                    for (int q = 0; q < io.e_parts; ++q) e += io.e_part[(base + k * L + i) * kPendParts + q];
                }
            }
        }
        l2nu[idx] = s;
        ex[idx] = e;
    }
    __syncthreads();
    // One entry of the acceptance table.  With may_mark (two-pass schedule, first visit): a row whose s and g cancel
    // so far that h needs E = nu^2 (s - g) summed term by term (the kernels' two tests; rows under pending
    // modifications keep the plain sum) is marked instead and true is returned; its entry is made after the
    // workgroups of the prefix have summed E together.
    auto table_entry = [&](int idx, bool may_mark) -> bool {
        const double e = philox_uniform(seed, offset, static_cast<uint32_t>(b), static_cast<uint32_t>(idx));
        if (idx == KL) { *u_final_out = e; return false; }
        const int k = idx / L, i = idx % L + 1;
        const double s = l2nu[idx];                         // parked by this thread above
        double log2nu = 0.0, log2P = 0.0;
        for (int j = 0; j < i; ++j) {
            log2nu += tq[k * L + j] - tp[k * L + j];
            log2P += tp[k * L + j];
        }
        const double log_nu = log2nu * kLn2, log_P = log2P * kLn2;
        // two exponentials per entry: 1/nu (nu by one division) and P
        const double inv_nu = exp2_small(-log2nu), P = exp2_small(log2P);
        const double nu = 1.0 / inv_nu;
        const double g = g_K(inv_nu, K), cK = c_K(P, K);
        double hv;
        if (i < L && log2nu > 0.0) {
            if (may_mark && excess_wanted(static_cast<float>(log2nu), static_cast<float>(s), K) &&
                excess_needed(log2nu, log2P, s, K)) {
                bool modified = false;
                if (io.pend)
                    for (int l = 0; l < io.nlev; ++l)
                        modified = modified || io.pend[static_cast<long long>(l) * io.n_rows + base + idx + 1].flag != 0;
                if (!modified) { ex[idx] = kExcessPending; return true; }
            }
            // Block ratio above one: the denominator c_K(P) - nu (1 - s) equals [c_K(P) - c_K(1/nu)] + nu (s - g),
            // and c_K(P) - c_K(1/nu) = (1 - Q) S2 / nu with Q = nu P the block's joint target probability and
            // S2 = sum_{j=1}^{K-1} sum_{m<j} (1-P)^m (1 - 1/nu)^(j-1-m) (by the recurrence U_1 = 1,
            // U_{j+1} = (1-P) U_j + (1 - 1/nu)^j), every term non-negative.  With E = nu^2 (s - g):
            // h = E / (E + (1 - Q) S2), where E comes from the sum kernels when s and g nearly cancel.
            const double A = 1.0 - P, t1 = 1.0 - inv_nu;
            double U = 1.0, S2 = 0.0, pw = 1.0;
            for (int j = 1; j <= K - 1; ++j) { S2 += U; pw *= t1; U = fma(A, U, pw); }
            const double one_Q = fmax(1.0 - exp2_small(log2nu + log2P), 0.0);
            const double E = ex[idx];
            if (E >= 0.0) {
                const double den = E + one_Q * S2;
                hv = !(E < 1.0e300) ? 1.0 : (den > 0.0 ? clamp01(E / den) : 1.0);
            } else {
                const double num = nu * (s - g);
                const double den = inv_nu * one_Q * S2 + num;
                hv = den > 0.0 ? clamp01(num / den) : 1.0;
            }
        } else if (i < L) {
            const double num = nu * (s - g);
            const double den = cK - nu * (1.0 - s);
            hv = den > 0.0 ? clamp01(num / den) : 1.0;
        } else {
            hv = clamp01(nu * (1.0 - g) / cK);
        }
        l2nu[idx] = log2nu;
        if (e < hv) atomicOr(&acc_bits[k], 1ull << i);
        if (write) {
            io.log_nu_out[base + idx] = log_nu; io.log_P_out[base + idx] = log_P;
            io.h_out[base + idx] = hv; io.eta_out[base + idx] = e;
        }
        return false;
    };
    unsigned marked = 0u;                                   // bit n: the entry of this thread's n-th visit was marked
    {
        int n = 0;
        for (int idx = tid; idx <= KL; idx += kDecideThreads, ++n)
            if (table_entry(idx, io.e_coop != 0)) marked |= 1u << n;
    }
    if (io.e_coop) {                                        // (uniform)
        static_assert((kMaxDrafts * 64 + kDecideThreads) / kDecideThreads <= 32, "one bit per visit (K <= 64, L < 64)");
        if (__syncthreads_or(marked != 0u)) {
            excess_sums(tq, tp, lq, lp, ex);
            int n = 0;
            for (int idx = tid; idx <= KL; idx += kDecideThreads, ++n)
                if (marked >> n & 1u) table_entry(idx, false);
        }
    }
    for (int idx = tid; idx < K * K; idx += kDecideThreads) {
        const int k1 = idx / K, k2 = idx % K;
        int n = 0;
        while (n < L && tok[k1 * L + n] == tok[k2 * L + n]) ++n;
        cpl[idx] = static_cast<unsigned char>(n);
    }
    __syncthreads();
    if (tid < kWave) {
    // Sequential loop of Algorithm 1, executed by the first wave.  acc_bits[j] holds the outcomes
    // of draft j's L tests as a bit mask (bit i: eta_{j,i} < h_{j,i}); lane j holds the lengths at
    // which draft j was tested and rejected (its entries of H) and its test states (2 bits per length: 1 tested,
    // 2 skipped because the block is in H).  For draft k the lengths already in H are the union
    // over earlier drafts j of (rejected_j restricted to lengths <= common prefix of j and k), a
    // wave-wide OR; the loop over lengths then runs on wave-uniform bit masks only.
    const int lane = tid;
    int tau = 0, f = -1;
    unsigned long long rejected = 0ull;
    unsigned long long st_lo = 0ull, st_hi = 0ull;        // state bits of draft `lane`
    bool done = false;
    // Per draft the loop over lengths has a closed form on bit masks, because the index keeps
    // running after an acceptance: every length in (tau, L] that is not in H is tested; the
    // longest accepted one becomes tau; the failed ones join H; a full-length acceptance ends
    // the scan.
    const unsigned long long upto_L = (2ull << L) - 1ull;                      // bits 0..L
    for (int k = 0; k < K && !done; ++k) {
        const int my_cpl = (lane < k) ? cpl[k * K + lane] : 0;
        const unsigned long long in_H =
            wave_or64((lane < k) ? (rejected & ((2ull << my_cpl) - 1ull)) : 0ull);   // lengths <= common prefix
        const unsigned long long acc_k = uniform_u64(acc_bits[k]);
        const unsigned long long range = upto_L & ~((2ull << tau) - 1ull);      // lengths tau+1 .. L
        const unsigned long long tested = range & ~in_H, skipped = range & in_H;
        const unsigned long long won = tested & acc_k;
        if (won) {
            tau = 63 - __clzll(static_cast<long long>(won));
            f = k;
            done = (won >> L) & 1ull;
        }
        if (lane == k) { st_lo = tested; st_hi = skipped; rejected = tested & ~acc_k; }
    }
    if (write && lane < K)
        for (int i = 1; i <= L; ++i)
            io.state_out[base + lane * L + i - 1] =
                static_cast<int32_t>(((st_lo >> i) & 1ull) | (((st_hi >> i) & 1ull) << 1));

    const int kf = f < 0 ? 0 : f;
    // the levels' entries of the selected row, one lane per level (independent loads instead of a serial walk)
    PendRow prl;
    prl.log2mu = 0.0; prl.log2N = 0.0; prl.tokadj = 0.0; prl.flag = 0; prl.pad = 0;
    if (io.pend && tau < L && lane < io.nlev) prl = io.pend[lane * io.n_rows + base + kf * L + tau];
    if (lane == 0) {
        if (write) {
            io.accepted_len[b] = tau;
            io.accepted_draft_idx[b] = f;
        }
        Selection &sl = *sel_out;                // built in place (LDS): the level constants are indexed at run time
        sl.tau = tau;
        sl.npend = 0; sl.C2_adj = 0.0f;
        tab_out->n = 0;
        sl.target_row = (static_cast<long long>(b) * K + kf) * (L + 1) + tau;
        if (tau == L) {
            sl.draft_row = -1; sl.C2 = 0.0; sl.shift_q = 0.0f; sl.lse2_q = 0.0; sl.lse2_pq = 0.0;
        } else {
            sl.draft_row = (static_cast<long long>(b) * K + kf) * L + tau;
            const double lse2_q = lq[kf * L + tau], lse2_p = lp[kf * L + tau];
            sl.C2 = lse2_p - lse2_q + (tau == 0 ? 0.0 : l2nu[kf * L + tau - 1]);
            const double adj = tau == 0 ? 0.0 : -io.c_rel * l2nu[kf * L + tau - 1];
            sl.C2_adj = adj - adj == 0.0 ? static_cast<float>(adj) : 0.0f;       // (an infinite block ratio stays what it is)
            sl.shift_q = rintf(static_cast<float>(lse2_q));         // integral: partial sums rescale exactly
            sl.lse2_q = lse2_q;
            sl.lse2_pq = lse2_p - lse2_q;
        }
    }
    // Levels that modify the selected row: q' = q prod t_l^K / N_l.  The whole wave walks the levels (tau, kf and
    // nlev are wave-uniform), so that every cross-lane read of the levels' entries happens with all lanes active
    // and outside any divergent branch; lane 0 alone patches the selection.
    if (io.pend && tau < L) {
        const double lse2_q = lq[kf * L + tau], lse2_p = lp[kf * L + tau];
        double sumN = 0.0;
        int n = 0;
        for (int l = 0; l < io.nlev; ++l) {
            const int flag_l = __builtin_amdgcn_readlane(prl.flag, l);
            const double mu_l = lane_value(prl.log2mu, l), N_l = lane_value(prl.log2N, l);
            if (flag_l) {
                const double Cl = lse2_p - lse2_q + mu_l - sumN;
                if (lane == 0) {
                    sel_out->Cl[n] = Cl;
                    pend_table_set(*tab_out, n, Cl);
                }
                ++n;
                sumN += N_l;
            }
        }
        if (lane == 0) {
            sel_out->npend = n;
            tab_out->n = n;
            sel_out->C2 -= sumN;
            sel_out->lse2_q = lse2_q + sumN;
        }
    }
    // position tau belongs to the final token, which the locating workgroup writes
    if (write)
        for (int j = lane; j <= L; j += kWave)
            if (j != tau) io.out_tokens[static_cast<long long>(b) * (L + 1) + j] = j < tau ? tok[kf * L + j] : -1;
    }
    __syncthreads();
}

// ------------------------------------------------- comparison verifier: the K-SEQ scan (Section 3.2)

// Decision of prefix b under the K-SEQ rule, by the whole workgroup; leaves the row the final token is drawn from
// in *sel_out (its weights max{q - rho p, 0} are the K = 1 residual weights at block ratio 1/rho) and the final
// uniform in *u_final_out.  For every (draft j, position i) the acceptance probability min{1, q(x)/(rho p(x))} of
// draft j's token is formed from the rows of the LEAD draft of j's first i tokens (the lowest draft that shares
// them: the drafts retained when the position is reached are exactly those sharing the accepted block), then one
// thread walks the positions on bit masks: the lowest retained draft whose test succeeds wins the position, and the
// drafts carrying its token stay retained.
template <typename T>
__device__ __forceinline__ void decide_kseq(const T *target, const T *draft, const DecideIO &io, int b, int K, int L, int V,
                                            float c, uint64_t seed, uint64_t offset, bool write, double *lds,
                                            Selection *sel_out, double *u_final_out, PendTable *tab_out)
{
    const int KL = K * L, nd = io.kseq_ndrafts;
    double *acc = lds;                                                          // [K*L] acceptance probabilities
    unsigned long long *eq = reinterpret_cast<unsigned long long *>(lds + KL);  // [K*L] drafts with draft j's token at position i
    unsigned long long *won = reinterpret_cast<unsigned long long *>(lds + 2 * KL);   // [L] drafts whose test at position i succeeds
    unsigned long long *tested = won + L;                                       // [L] drafts tested at position i
    int *lead_of = reinterpret_cast<int *>(tested + L);                         // [K*L] (in all 3 K L + 2 L doubles of the 6 K L + K)
    int *tok = lead_of + KL;                                                    // [K*L]
    const int tid = threadIdx.x;
    const long long base = static_cast<long long>(b) * KL;
    for (int idx = tid; idx < KL; idx += kDecideThreads) tok[idx] = io.tokens[base + idx];
    for (int idx = tid; idx < L; idx += kDecideThreads) { won[idx] = 0ull; tested[idx] = 0ull; }
    __syncthreads();
    for (int idx = tid; idx <= KL; idx += kDecideThreads) {
        if (idx == KL) { *u_final_out = philox_uniform(seed, offset, static_cast<uint32_t>(b), static_cast<uint32_t>(KL)); continue; }
        const int j = idx / L, i = idx % L;
        double a = 0.0, e = 0.0;
        unsigned long long same_tok = 0ull;
        int lead = j;
        if (j < nd) {
            for (int m = j - 1; m >= 0; --m) {                                  // lowest draft sharing the first i tokens
                bool same = true;
                for (int q = 0; q < i; ++q) same = same && tok[m * L + q] == tok[j * L + q];
                if (same) lead = m;
            }
            for (int m = 0; m < nd; ++m) same_tok |= static_cast<unsigned long long>(tok[m * L + i] == tok[j * L + i]) << m;
            int x = tok[idx];
            x = x < 0 ? 0 : (x >= V ? V - 1 : x);
            const long long lrow = (static_cast<long long>(b) * K + lead) * L + i;
            const RowStat st = io.stats[lrow];
            const double zq = static_cast<double>(Elem<T>::scalar(target + ((static_cast<long long>(b) * K + lead) * (L + 1) + i) * V + x));
            const double zp = static_cast<double>(Elem<T>::scalar(draft + lrow * V + x));
            const double l2 = ((static_cast<double>(c) * zq - st.lse2_q) - (static_cast<double>(c) * zp - st.lse2_p)) * (1.0 + io.c_rel);
            const double ratio = exp2_small(l2) / io.s_arr[lrow];               // q(x) / (rho p(x))
            a = ratio < 1.0 ? ratio : 1.0;
            e = philox_uniform(seed, offset, static_cast<uint32_t>(b), static_cast<uint32_t>(idx));
            if (e < a) atomicOr(&won[i], 1ull << j);
        }
        acc[idx] = a; eq[idx] = same_tok; lead_of[idx] = lead;
        if (write) { io.h_out[base + idx] = a; io.eta_out[base + idx] = e; }
    }
    __syncthreads();
    if (tid == 0) {
        unsigned long long alive = nd >= 64 ? ~0ull : ((1ull << nd) - 1ull);
        int tau = 0;
        for (int i = 0; i < L; ++i) {
            const int lead = __ffsll(static_cast<long long>(alive)) - 1;
            if (write) {
                io.kseq_pos[static_cast<long long>(b) * L + i] = __popcll(alive);
                io.kseq_pos[static_cast<long long>(gridDim.y) * L + static_cast<long long>(b) * L + i] = lead;
            }
            const unsigned long long cand = alive & won[i];
            if (!cand) { tested[i] = alive; break; }
            const int w = __ffsll(static_cast<long long>(cand)) - 1;
            tested[i] = alive & ((2ull << w) - 1ull);
            alive &= eq[w * L + i];
            tau = i + 1;
        }
        if (write)
            for (int i = tau + 1; i < L; ++i) {                                  // positions never reached
                io.kseq_pos[static_cast<long long>(b) * L + i] = 0;
                io.kseq_pos[static_cast<long long>(gridDim.y) * L + static_cast<long long>(b) * L + i] = -1;
            }
        const int lead = __ffsll(static_cast<long long>(alive)) - 1;
        Selection &sl = *sel_out;
        sl.tau = tau; sl.npend = 0; sl.C2_adj = 0.0f; tab_out->n = 0;
        sl.target_row = (static_cast<long long>(b) * K + lead) * (L + 1) + tau;
        if (tau == L) {
            sl.draft_row = -1; sl.C2 = 0.0; sl.shift_q = 0.0f; sl.lse2_q = 0.0; sl.lse2_pq = 0.0;
        } else {
            const long long lrow = (static_cast<long long>(b) * K + lead) * L + tau;
            const RowStat st = io.stats[lrow];
            sl.draft_row = lrow;
            sl.C2 = st.lse2_p - st.lse2_q - log2(io.s_arr[lrow]);                // rho p / q = 2^(c (z_p - z_q) - C2)
            sl.shift_q = rintf(static_cast<float>(st.lse2_q));
            sl.lse2_q = st.lse2_q;
            sl.lse2_pq = st.lse2_p - st.lse2_q;
        }
        if (write) {
            io.accepted_len[b] = tau;
            io.accepted_draft_idx[b] = tau > 0 ? lead : -1;
            for (int j = 0; j <= L; ++j)
                if (j != tau) io.out_tokens[static_cast<long long>(b) * (L + 1) + j] = j < tau ? tok[lead * L + j] : -1;
        }
    }
    __syncthreads();
    if (write)
        for (int idx = tid; idx < KL; idx += kDecideThreads)
            io.state_out[base + idx] = static_cast<int32_t>((tested[idx % L] >> (idx / L)) & 1ull);
    __syncthreads();
}

// ------------------------------------------------------------ final token

// The 8 logits [e0, e0+8) of a row; entries at or beyond V read as -inf.
template <typename T, bool VEC>
__device__ __forceinline__ void load8(const T *row, long long e0, int V, float (&z)[8])
{
    constexpr int PV = Elem<T>::kPerVec;
    if (VEC && e0 + 8 <= V) {
#pragma unroll
        for (int v = 0; v < 8 / PV; ++v) {
            float t[PV];
            Elem<T>::unpack(load16(row + e0 + v * PV), t);
#pragma unroll
            for (int j = 0; j < PV; ++j) z[v * PV + j] = t[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) z[j] = (e0 + j < V) ? Elem<T>::scalar(row + e0 + j) : -INFINITY;
    }
}

// This lane's 8 logits of segment `seg` from the target row and (unless the bonus row is
// drawn from) the draft row; entries at or beyond V read as -inf / 0.
template <typename T, bool VEC>
__device__ __forceinline__ void segment_load(const T *target, const T *draft, const Selection &sl, int V, int seg,
                                             int lane, float (&zq)[8], float (&zp)[8])
{
    const long long e0 = static_cast<long long>(seg) * kSegElems + lane * 8;
    if (e0 < V) load8<T, VEC>(target + sl.target_row * V, e0, V, zq);
    else {
#pragma unroll
        for (int j = 0; j < 8; ++j) zq[j] = -INFINITY;
    }
    if (sl.draft_row >= 0 && e0 < V) load8<T, VEC>(draft + sl.draft_row * V, e0, V, zp);
    else {
#pragma unroll
        for (int j = 0; j < 8; ++j) zp[j] = 0.0f;
    }
}

// Weights of this lane's 8 entries of segment `seg` relative to 2^m2 (w: the weights the
// token is drawn from; wq: plain target weights).  With m2 = NaN on entry for the bonus row
// the segment's own maximum is used as reference and returned.
template <bool PEND>
__device__ __forceinline__ float segment_weigh(const Selection &sl, const PendTable &tab, int V, int K, float c, int seg,
                                               int lane, float m2_in, const float (&zq)[8], const float (&zp)[8],
                                               float (&w)[8], float (&wq)[8])
{
    const long long e0 = static_cast<long long>(seg) * kSegElems + lane * 8;
    if (sl.draft_row < 0) {
        float m2 = m2_in;
        if (!(m2 == m2)) {                      // reference not fixed yet: this segment's maximum
            float m = -3.0e38f;
#pragma unroll
            for (int j = 0; j < 8; ++j) m = fmaxf(m, zq[j]);
            m2 = integral_reference(wave_max(m), c);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) { wq[j] = exp2_fast(fmaf(zq[j], c, -m2)); w[j] = wq[j]; }
        return m2;
    }
    const float m2 = sl.shift_q;
    const RatioConst rc(sl.C2 + static_cast<double>(sl.C2_adj));
    if (PEND && tab.n > 0) {
        // modified row: plain weights q prod t_l^K, residual weights those times max(1 - p/(nu q'), 0)^K
        pending_weights(zq, zp, c, m2, tab, rc, K, wq, w);
    } else {
        ot_weights(zq, zp, c, m2, rc, K, wq, w);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (!(e0 + j < V)) { wq[j] = 0.0f; w[j] = 0.0f; }
    return m2;
}

// Partial sums travel between workgroups of one kernel, possibly on different dies with
// separate L2 caches: they are written and read with device-scope relaxed atomic accesses
// (which bypass the non-coherent cache levels) instead of being published with a device-scope
// fence, which on this hardware writes back the whole L2 and costs microseconds per wave.
__device__ __forceinline__ void partial_store(SegPartial *dst, double sum_w, double sum_q, float m2)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(&dst->sum_w), static_cast<unsigned long long>(__double_as_longlong(sum_w)),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(&dst->sum_q), static_cast<unsigned long long>(__double_as_longlong(sum_q)),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<unsigned *>(&dst->m2), __float_as_uint(m2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double partial_load_d(const double *src)
{
    return __longlong_as_double(static_cast<long long>(__hip_atomic_load(
        reinterpret_cast<const unsigned long long *>(src), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
}
__device__ __forceinline__ float partial_load_m2(const SegPartial *src)
{
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned *>(&src->m2), __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT));
}

struct FinalOut {
    Selection *sel;              // [batch] what the final token of each prefix is drawn from (kept for inspection)
    SegPartial *partial;         // [batch, nseg]
    int32_t *counter;            // [batch] workgroups of the prefix that have stored their partial sums
    double *res_norm, *u_final, *margin;
    int32_t *fallback;
    double *carry;
    int32_t *mcount;
    double *state_carry;         // pending state updated in place ([kMaxPend][batch] each), or null
    int32_t *state_count;
};

// Sum over aligned groups of 4 lanes (every lane of a group gets its group's sum).
__device__ __forceinline__ double group4_sum(double v)
{
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    return v;
}

// Algorithm 3's bookkeeping for prefix b after its final token is known, by the whole first wave of
// the locating workgroup: every pending level's block ratio is continued along the tokens this
// iteration emitted (draft f's tokens 0 .. tau-1, then the final token y), with the token
// probabilities under the distribution THAT level modifies (the target rows as the levels below it
// left them); its row count shrinks by tau + 1; used-up levels are dropped, the others move down,
// and the modification this iteration creates (carry_new, count_new) is appended.  Lanes 4 m .. 4 m + 3
// look after level m (at most kMaxPend = 16 levels), lane 4 m + q after its emitted rows j = q, q + 4, ...
template <typename T>
__device__ __forceinline__ void update_pending_state(const T *target, const T *draft, const DecideIO &io, const FinalOut &fo,
                                                     const Selection &sl, int b, int K, int L, int V, float c, int winner,
                                                     int tokid_w, double carry_w, int mcount_w)
{
    static_assert(kMaxPend * 4 == kWave, "four lanes per level");
    constexpr double kLn2 = 0.693147180559945309417;
    const int lane = threadIdx.x & (kWave - 1);
    const int m = lane >> 2, q = lane & 3;
    const int nlev = io.nlev, tau = sl.tau;
    const int batch = static_cast<int>(gridDim.y);
    const int tokid = __builtin_amdgcn_readlane(tokid_w, winner);
    const int count_new = __builtin_amdgcn_readlane(mcount_w, winner);
    const double carry_new = lane_value(carry_w, winner);
    // old state of level m (read by every lane of its group before anything is written)
    int count_m = 0;
    double carry_m = 0.0;
    if (m < nlev) { count_m = fo.state_count[static_cast<size_t>(m) * batch + b]; carry_m = fo.state_carry[static_cast<size_t>(m) * batch + b]; }
    double val = 0.0;            // what level m does to the log2 probability of the tokens emitted at this lane's rows
    double base = 0.0;           // log2 q_j[e_j] - log2 p_j[e_j] under the unmodified rows, row j = lane
    const bool some_may_survive = tau + 2 <= L - 1;   // a level survives only if tau + 1 < count <= L - 1
    if (some_may_survive) {      // uniform; otherwise (in particular after a whole accepted block) every level ends
        const int kf = static_cast<int>(sl.draft_row / L - static_cast<long long>(b) * K);
        const long long row0 = (static_cast<long long>(b) * K + kf) * L;
        // accepted draft tokens: rows j < tau
        if (m < nlev)
            for (int j = q; j < tau; j += 4) {
                const PendRow pr = io.pend[m * io.n_rows + row0 + j];
                val += pr.tokadj - pr.log2N;
            }
        if (lane < tau) {
            const RowStat st = io.stats[row0 + lane];
            base = (st.tok2_q - st.lse2_q) - (st.tok2_p - st.lse2_p);
        }
        // the final token y at row tau: its probabilities under the unmodified rows ...
        const RowStat st_tau = io.stats[row0 + tau];
        const double zq_y = static_cast<double>(Elem<T>::scalar(target + sl.target_row * V + tokid)) * static_cast<double>(c);
        const double zp_y = static_cast<double>(Elem<T>::scalar(draft + sl.draft_row * V + tokid)) * static_cast<double>(c);
        const double by = ((zq_y - st_tau.lse2_q) - (zp_y - st_tau.lse2_p)) * (1.0 + io.c_rel);
        if (lane == tau) base = by;
        // ... and the levels' factors there, one level after the other (wave-uniform loop; lane 4 l holds level l's entry)
        PendRow pt;
        pt.log2mu = 0.0; pt.log2N = 0.0; pt.tokadj = 0.0; pt.flag = 0; pt.pad = 0;
        if (m < nlev && q == 0) pt = io.pend[m * io.n_rows + row0 + tau];
        double log2T = 0.0, sumN = 0.0;
        for (int l = 0; l < nlev; ++l) {
            const int src = l * 4;
            if (!__builtin_amdgcn_readlane(pt.flag, src)) continue;
            const double log2mu = lane_value(pt.log2mu, src), log2N = lane_value(pt.log2N, src);
            const double t = 1.0 - exp2_small(-by - log2mu + sumN - log2T);        // 1 - p[y] / (mu_l q^(l)[y])
            const double adj = t > 0.0 ? static_cast<double>(K) * log2(t) : -INFINITY;
            if (lane == src) val += adj - log2N;
            log2T += adj;
            sumN += log2N;
        }
    }
    const double S = group4_sum(val);                        // level m: sum over the emitted rows
    const double B = wave_sum(base);                         // unmodified rows
    // levels in order: the ratio of level l moves by B plus what the levels below it contribute
    double run = B;
    int pos = 0;
    for (int l = 0; l < nlev; ++l) {
        const int cnt = __builtin_amdgcn_readlane(count_m, l * 4);
        const double car = lane_value(carry_m, l * 4);
        if (some_may_survive && cnt > tau + 1) {
            if (lane == 0) {
                fo.state_carry[static_cast<size_t>(pos) * batch + b] = car + run * kLn2;
                fo.state_count[static_cast<size_t>(pos) * batch + b] = cnt - (tau + 1);
            }
            ++pos;
        }
        run += lane_value(S, l * 4);
    }
    if (count_new > 0 && pos < kMaxPend) {
        if (lane == 0) {
            fo.state_carry[static_cast<size_t>(pos) * batch + b] = carry_new;
            fo.state_count[static_cast<size_t>(pos) * batch + b] = count_new;
        }
        ++pos;
    }
    if (lane >= pos && lane < kMaxPend) {
        fo.state_carry[static_cast<size_t>(lane) * batch + b] = 0.0;
        fo.state_count[static_cast<size_t>(lane) * batch + b] = 0;
    }
}

template <typename T, bool VEC, bool PEND>
__global__ void __launch_bounds__(kSegThreads)
k_final(const T *__restrict__ target, const T *__restrict__ draft, DecideIO io, FinalOut fo, int V, int K, int L,
        float c, int nseg, uint64_t seed, uint64_t offset)
{
    static_assert(kSegThreads == kDecideThreads, "the decision runs on the whole workgroup");
    extern __shared__ double lds_decide[];
    __shared__ Selection sh_sel;
    __shared__ PendTable sh_tab;
    __shared__ double sh_u;
    __shared__ int sh_is_last;
    __shared__ double sh_d[kSegThreads / kWave];
    __shared__ double sh_scan[kSegThreads / kWave];
    __shared__ float sh_f[kSegThreads / kWave];
    __shared__ int sh_seg, sh_first[kSegThreads / kWave], sh_last[kSegThreads / kWave];
    __shared__ double sh_local_target, sh_total;
    __shared__ float sh_seg_m2;
    __shared__ double sh_excess[kPendParts];
    const int b = blockIdx.y, tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wid = tid / kWave;
    int32_t *__restrict__ out_tokens = io.out_tokens;
    double *__restrict__ res_norm = fo.res_norm, *__restrict__ u_final = fo.u_final, *__restrict__ margin_out = fo.margin;
    int32_t *__restrict__ fallback_out = fo.fallback, *__restrict__ mcount_out = fo.mcount;
    double *__restrict__ carry_out = fo.carry;

    // ---- 1. decision (redundantly per workgroup; the first one of the prefix writes it out)
    if (io.kseq_ndrafts > 0) {             // comparison verifier: K-SEQ scan; its replacement weights are the K = 1 ones
        decide_kseq<T>(target, draft, io, b, K, L, V, c, seed, offset, blockIdx.x == 0, lds_decide, &sh_sel, &sh_u, &sh_tab);
        K = 1;
    } else {
        // Two-pass schedule: whether a row's s and g cancel so far that its E = nu^2 (s - g) has to be summed term by
        // term is looked at here (with small batches the sums of Eq. (hik) arrive in parts and meet here; with larger
        // ones the sum kernel's workgroup would have to take a second sweep alone).  tq holds the token probabilities
        // under the pending modifications, if there are any, so nu is the one the decision uses.  Every workgroup of the
        // prefix applies the kernels' two tests to every row while it makes the acceptance table (the same values, so
        // the same rows), and for the rare row that fails them the workgroups sum E together, straight from memory (this
        // function, called only then): one part per workgroup (at most
        // kPendParts), left in the workspace with a device-scope store; every workgroup needs all parts (each runs the
        // decision itself) and polls for the ones it has not summed.  The wait is bounded: a part that has not
        // arrived after io.e_polls looks (its workgroup has not been scheduled yet, say) is summed by the waiting
        // workgroup itself -- the same bits, stored again -- so no workgroup depends on another one's progress.
        auto excess_sums = [&](const double *tq, const double *tp, const double *lq, const double *lp, double *ex) {
            const int KL = K * L;
            constexpr int N = VEC ? Elem<T>::kPerVec : 1;
            constexpr int kAhead = 4;                                  // vector pairs in flight per thread
            const int nparts = static_cast<int>(gridDim.x) < kPendParts ? static_cast<int>(gridDim.x) : kPendParts;
            const int units = VEC ? V / N : V;
            const int per = (units + nparts - 1) / nparts;
            for (int idx = 0; idx < KL; ++idx) {                       // uniform: every thread reads the same LDS entry
                if (ex[idx] != kExcessPending) continue;
                const int k = idx / L, i = idx % L + 1;
                const long long bk = static_cast<long long>(b) * K + k, pair = bk * L + i;
                double log2nu = 0.0;
                for (int j = 0; j < i; ++j) log2nu += tq[k * L + j] - tp[k * L + j];
                const ExcessConst ec = make_excess_const(lq[k * L + i], lp[k * L + i], log2nu, K, c);
                const T *rq = target + (bk * (L + 1) + i) * static_cast<long long>(V);
                const T *rp = draft + pair * static_cast<long long>(V);
                double *parts = io.e_part_rw + pair * kPendParts;
                auto sum_part = [&](int part) {                        // by the whole workgroup; the value in every thread
                    const int lo = part * per, hi = lo + per < units ? lo + per : units;
                    float acc = 0.0f;
                    if constexpr (VEC) {
                        for (int v0 = lo + tid; v0 < hi; v0 += kAhead * kSegThreads) {
                            U4 q4[kAhead], p4[kAhead];
#pragma unroll
                            for (int a = 0; a < kAhead; ++a) {
                                const int v = v0 + a * kSegThreads;
                                q4[a] = load16_stream(rq + static_cast<long long>(v < hi ? v : v0) * N);
                                p4[a] = load16_stream(rp + static_cast<long long>(v < hi ? v : v0) * N);
                            }
#pragma unroll
                            for (int a = 0; a < kAhead; ++a) {
                                float zq[N], zp[N];
                                Elem<T>::unpack(q4[a], zq);
                                Elem<T>::unpack(p4[a], zp);
                                if (v0 + a * kSegThreads < hi) acc += excess_terms(zq, zp, ec);
                            }
                        }
                    } else {
                        for_each_pair_range<T, VEC, kSegThreads>(rq, rp, lo, hi, [&](int, const float (&zq)[N], const float (&zp)[N]) {
                            acc += excess_terms(zq, zp, ec);
                        });
                    }
                    const double v = block_sum(static_cast<double>(acc), sh_d) * ec.scale;
                    if (tid == 0)
                        __hip_atomic_store(reinterpret_cast<unsigned long long *>(parts + part),
                                           static_cast<unsigned long long>(__double_as_longlong(v)), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    return v;
                };
                __syncthreads();                                       // (sh_excess of the previous row has been read)
                {
                    const int mine = static_cast<int>(blockIdx.x);     // (workgroups beyond kPendParts only wait)
                    const double v = mine < nparts ? sum_part(mine) : -1.0;
                    if (tid < kPendParts) sh_excess[tid] = tid == mine ? v : -1.0;
                }
                __syncthreads();
                if (tid < nparts && sh_excess[tid] == -1.0) {
                    double v = -1.0;
                    for (int look = 0; look < io.e_polls && v == -1.0; ++look) {
                        v = partial_load_d(parts + tid);
                        if (v == -1.0) __builtin_amdgcn_s_sleep(8);
                    }
                    sh_excess[tid] = v;
                }
                __syncthreads();
                for (int part = 0; part < nparts; ++part) {            // uniform; normally none is missing
                    if (sh_excess[part] == -1.0) {
                        const double v = sum_part(part);
                        __syncthreads();
                        if (tid == 0) sh_excess[part] = v;
                        __syncthreads();
                    }
                }
                if (tid == 0) {
                    double e = 0.0;
                    for (int part = 0; part < nparts; ++part) e += sh_excess[part];          // in part order
                    ex[idx] = e;
                }
                __syncthreads();
            }
        };
        decide_prefix(io, b, K, L, seed, offset, blockIdx.x == 0, lds_decide, &sh_sel, &sh_u, &sh_tab, excess_sums);
    }
    const Selection sl = sh_sel;
    if (blockIdx.x == 0 && tid == 0) fo.sel[b] = sl;

    // ---- 2. partial sums of this workgroup's segments: kSegPerWave consecutive segments per wave
    {
        const int seg0 = (blockIdx.x * (kSegThreads / kWave) + wid) * kSegPerWave;
        double sw[kSegPerWave], sq[kSegPerWave];
        float m2[kSegPerWave];
        float zq[kSegPerWave][8], zp[kSegPerWave][8];
#pragma unroll
        for (int i = 0; i < kSegPerWave; ++i)            // all loads first: one memory latency, not four
            if (seg0 + i < nseg) segment_load<T, VEC>(target, draft, sl, V, seg0 + i, lane, zq[i], zp[i]);
#pragma unroll
        for (int i = 0; i < kSegPerWave; ++i) {
            sw[i] = 0.0; sq[i] = 0.0; m2[i] = 0.0f;
            if (seg0 + i < nseg) {                      // wave-uniform
                float w[8], wq[8];
                m2[i] = segment_weigh<PEND>(sl, sh_tab, V, K, c, seg0 + i, lane, __builtin_nanf(""), zq[i], zp[i], w, wq);
#pragma unroll
                for (int j = 0; j < 8; ++j) { sw[i] += static_cast<double>(w[j]); sq[i] += static_cast<double>(wq[j]); }
            }
        }
#pragma unroll
        for (int i = 0; i < kSegPerWave; ++i) {
            if (seg0 + i < nseg) {
                const double a = wave_sum(sw[i]), bq = wave_sum(sq[i]);
                if (lane == 0) partial_store(&fo.partial[static_cast<long long>(b) * nseg + seg0 + i], a, bq, m2[i]);
            }
        }
    }
    // ---- 3. the last workgroup of the prefix to get here locates the token.  The partial
    // stores above are device-scope accesses; the workgroup-scope release fence waits until
    // they have completed, the barrier orders them before the first thread's counter update.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
        const int arrived = __hip_atomic_fetch_add(&fo.counter[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_is_last = arrived == static_cast<int>(gridDim.x) - 1;
    }
    __syncthreads();
    if (!sh_is_last) return;
    const SegPartial *pp = fo.partial + static_cast<long long>(b) * nseg;

    // thread t owns the contiguous segments [t*chunk, (t+1)*chunk); the first kKeep of them stay
    // in registers (all of them up to V = 256K), later ones are read again when needed
    constexpr int kKeep = 2;
    const int chunk = (nseg + kSegThreads - 1) / kSegThreads;
    const int s0 = tid * chunk, s1 = min(nseg, s0 + chunk);
    float km2[kKeep];
    double kw[kKeep], kq[kKeep];
    float mloc = -3.0e38f;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        km2[i] = -3.0e38f; kw[i] = 0.0; kq[i] = 0.0;
        if (s0 + i < s1) {
            km2[i] = partial_load_m2(&pp[s0 + i]);
            kw[i] = partial_load_d(&pp[s0 + i].sum_w); kq[i] = partial_load_d(&pp[s0 + i].sum_q);
            mloc = fmaxf(mloc, km2[i]);
        }
    }
    for (int s = s0 + kKeep; s < s1; ++s) mloc = fmaxf(mloc, partial_load_m2(&pp[s]));
    const float M = block_max(mloc, sh_f);
    double tw = 0.0, tqs = 0.0;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        if (s0 + i < s1) {
            const int sh = reference_shift(km2[i], M);                         // both integral, difference <= 0
            kw[i] = ldexp(kw[i], sh); kq[i] = ldexp(kq[i], sh);               // now relative to 2^M
            tw += kw[i]; tqs += kq[i];
        }
    }
    for (int s = s0 + kKeep; s < s1; ++s) {
        const int sh = reference_shift(partial_load_m2(&pp[s]), M);
        tw += ldexp(partial_load_d(&pp[s].sum_w), sh); tqs += ldexp(partial_load_d(&pp[s].sum_q), sh);
    }
    const double Ww = block_sum(tw, sh_d);
    const double Wq = block_sum(tqs, sh_d);
    const bool use_q = !(Ww > 0.0);           // every residual weight is zero: draw from q
    const double W = use_q ? Wq : Ww;
    const double u = sh_u;
    const double goal = u * W;

    // first thread, then first segment, whose running total exceeds the goal
    const double mine_seg = use_q ? tqs : tw;
    const double incl_t = wave_inclusive_sum(mine_seg);
    if (lane == kWave - 1) sh_scan[wid] = incl_t;
    __syncthreads();
    double wave_off = 0.0;
    for (int wv = 0; wv < wid; ++wv) wave_off += sh_scan[wv];
    const double excl_t = wave_off + incl_t - mine_seg;
    // per wave: first thread whose running total exceeds the goal, last thread with any weight
    // (ballots; same-address LDS atomics from every lane serialise and cost microseconds)
    const unsigned long long has = __ballot(mine_seg > 0.0);
    const unsigned long long over = __ballot(mine_seg > 0.0 && excl_t + mine_seg > goal);
    if (lane == 0) {
        sh_first[wid] = over ? wid * kWave + __ffsll(static_cast<long long>(over)) - 1 : kSegThreads;
        sh_last[wid] = has ? wid * kWave + 63 - __clzll(static_cast<long long>(has)) : -1;
    }
    __syncthreads();
    int win_t = kSegThreads, last_t = -1;
#pragma unroll
    for (int wv = 0; wv < kSegThreads / kWave; ++wv) { win_t = min(win_t, sh_first[wv]); last_t = max(last_t, sh_last[wv]); }
    if (win_t == kSegThreads) win_t = last_t < 0 ? 0 : last_t;   // rounding pushed the goal past the end
    __syncthreads();
    if (tid == win_t) {
        double cum = excl_t, cum_before = excl_t;
        int found = -1, last_pos = s0 < nseg ? s0 : 0;
        float found_m2 = km2[0], last_m2 = km2[0];
        double cum_before_last = excl_t;
        bool open = true;
#pragma unroll
        for (int i = 0; i < kKeep; ++i) {
            if (open && s0 + i < s1) {
                const double v = use_q ? kq[i] : kw[i];
                if (v > 0.0) { last_pos = s0 + i; last_m2 = km2[i]; cum_before_last = cum; }
                if (cum + v > goal) { found = s0 + i; found_m2 = km2[i]; cum_before = cum; open = false; }
                else cum += v;
            }
        }
        for (int s = s0 + kKeep; open && s < s1; ++s) {
            const float m2s = partial_load_m2(&pp[s]);
            const double v = ldexp(partial_load_d(use_q ? &pp[s].sum_q : &pp[s].sum_w), reference_shift(m2s, M));
            if (v > 0.0) { last_pos = s; last_m2 = m2s; cum_before_last = cum; }
            if (cum + v > goal) { found = s; found_m2 = m2s; cum_before = cum; open = false; }
            else cum += v;
        }
        if (found < 0) { found = last_pos; found_m2 = last_m2; cum_before = cum_before_last; }
        const int up = -reference_shift(found_m2, M);
        sh_seg = found;
        sh_seg_m2 = found_m2;
        sh_local_target = ldexp(goal - cum_before, up);    // goal in the segment's own scale
        sh_total = ldexp(W, up);
    }
    __syncthreads();
    if (wid != 0) return;

    // inside the segment: one wave, lane order = token-id order
    const int seg = sh_seg;
    const double local_target = sh_local_target;
    float w[8], wq[8];
    {
        float zq[8], zp[8];
        segment_load<T, VEC>(target, draft, sl, V, seg, lane, zq, zp);
        segment_weigh<PEND>(sl, sh_tab, V, K, c, seg, lane, sh_seg_m2, zq, zp, w, wq);
    }
    double ws[8];
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        ws[j] = static_cast<double>(use_q ? wq[j] : w[j]);
        mine += ws[j];
    }
    const double incl = wave_inclusive_sum(mine);
    const double excl = incl - mine;
    const unsigned long long cross = __ballot(mine > 0.0 && incl > local_target);
    const unsigned long long pos = __ballot(mine > 0.0);
    int winner;
    if (cross) winner = __ffsll(static_cast<long long>(cross)) - 1;
    else if (pos) winner = 63 - __clzll(static_cast<long long>(pos));
    else winner = 0;
    int tokid_w = 0, mcount_w = 0;               // the winner lane's results, for the state update below
    double carry_w = 0.0;
    if (lane == winner) {
        const long long e0 = static_cast<long long>(seg) * kSegElems + lane * 8;
        double run = excl;
        int y = -1;
        double mg = 0.0;
        int last = -1;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double prev = run;
            run += ws[j];
            if (ws[j] > 0.0) last = j;
            if (y < 0 && run > local_target) {
                y = j;
                const double lo = local_target - prev, hi = run - local_target;
                mg = (lo < hi ? lo : hi) / sh_total;
            }
        }
        if (y < 0) { y = last < 0 ? 0 : last; mg = 0.0; }
        long long tokid = e0 + y;
        if (tokid >= V) tokid = V - 1;
        out_tokens[static_cast<long long>(b) * (L + 1) + sl.tau] = static_cast<int32_t>(tokid);
        margin_out[b] = mg;
        u_final[b] = u;
        fallback_out[b] = use_q ? 1 : 0;
        // total weight in probability units: weights are relative to 2^M, the target row's
        // normaliser is 2^lse2_q (bonus row: the total is the normaliser itself)
        res_norm[b] = sl.draft_row < 0 ? 1.0 : W * exp2_small(static_cast<double>(M) - sl.lse2_q);
        // Algorithm 2 conditions the next iteration on (t^tau, y): the block ratio extended by
        // the final token, ln [nu_tau q_tau[y] / p_tau[y]], and the number of rows it modifies
        double carry = 0.0;
        if (sl.draft_row >= 0) {
            const double zq = static_cast<double>(Elem<T>::scalar(target + sl.target_row * V + tokid));
            const double zp = static_cast<double>(Elem<T>::scalar(draft + sl.draft_row * V + tokid));
            double l2 = sl.C2 + static_cast<double>(c) * (zq - zp);        // log2 of nu_tau q[y] / p[y]
            // y's two log-probabilities at the caller's temperature (token_scaled); p[y] = 0 leaves the ratio infinite
            const double adj = static_cast<double>(c) * (zq - zp) + sl.lse2_pq;
            if (adj - adj == 0.0) l2 += io.c_rel * adj;
            if (PEND) {                                     // q'[y] = q[y] prod_l t_l[y]^K / N_l (the N_l are in C2)
                double log2T = 0.0;
                for (int l = 0; l < sl.npend; ++l) {
                    const double t = 1.0 - exp2_small(static_cast<double>(c) * (zp - zq) - sh_sel.Cl[l] - log2T);   // (LDS: run-time index)
                    log2T = t > 0.0 ? log2T + static_cast<double>(K) * log2(t) : -INFINITY;
                }
                l2 += log2T;
            }
            carry = l2 * 0.693147180559945309417;
        }
        carry_out[b] = carry;
        mcount_out[b] = sl.draft_row < 0 ? 0 : L - sl.tau - 1;
        tokid_w = static_cast<int>(tokid); carry_w = carry; mcount_w = sl.draft_row < 0 ? 0 : L - sl.tau - 1;
    }
    if (PEND && fo.state_carry) update_pending_state<T>(target, draft, io, fo, sl, b, K, L, V, c, winner, tokid_w, carry_w, mcount_w);
}

template <typename T>
hipError_t launch_final_typed(const Problem &p)
{
    const T *target = static_cast<const T *>(p.target);
    const T *draft = static_cast<const T *>(p.draft);
    const bool vec = (p.V % Elem<T>::kPerVec) == 0 &&
                     (reinterpret_cast<uintptr_t>(p.target) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(p.draft) % 16 == 0);
    constexpr int kSegPerBlock = kSegThreads / kWave * kSegPerWave;
    const dim3 g(static_cast<unsigned>((p.lay.nseg + kSegPerBlock - 1) / kSegPerBlock), static_cast<unsigned>(p.batch));
    DecideIO io;
    io.tokens = p.tokens;
    io.stats = reinterpret_cast<const RowStat *>(p.ws + p.lay.stats);
    io.pend = p.pend_levels > 0 ? reinterpret_cast<const PendRow *>(p.ws + p.lay.pend) : nullptr;
    io.n_rows = static_cast<long long>(p.batch) * p.K * p.L;
    io.nlev = p.pend_levels;
    io.s_arr = reinterpret_cast<const double *>(p.ws + p.lay.s);
    io.e_arr = reinterpret_cast<const double *>(p.ws + p.lay.excess);
    io.e_part = reinterpret_cast<const double *>(p.ws + p.lay.excess_part);
    io.s_part = reinterpret_cast<const double *>(p.ws + p.lay.pend_part);
    io.s_store = reinterpret_cast<double *>(p.ws + p.lay.s);
    io.s_parts = p.s_parts;
    io.e_parts = p.e_parts;
    io.e_coop = (p.e_coop != 0 && p.kseq_ndrafts == 0) ? 1 : 0;
    io.e_part_rw = reinterpret_cast<double *>(p.ws + p.lay.excess_part);
    // (the environment variable lets a test take the fall-back of the bounded wait: 0 looks, every workgroup sums all parts)
    io.e_polls = 1024;
    if (const char *polls = std::getenv("SPECGBV_EXCESS_POLLS")) {
        const long n = std::strtol(polls, nullptr, 10);
        io.e_polls = n < 0 ? 0 : (n > 1048576 ? 1048576 : static_cast<int>(n));
    }
    io.log_nu_out = reinterpret_cast<double *>(p.ws + p.lay.log_nu);
    io.log_P_out = reinterpret_cast<double *>(p.ws + p.lay.log_P);
    io.h_out = reinterpret_cast<double *>(p.ws + p.lay.h);
    io.eta_out = reinterpret_cast<double *>(p.ws + p.lay.eta);
    io.state_out = reinterpret_cast<int32_t *>(p.ws + p.lay.state);
    io.accepted_len = p.accepted_len; io.accepted_draft_idx = p.accepted_draft_idx; io.out_tokens = p.out_tokens;
    io.c_rel = p.c_rel;
    io.kseq_ndrafts = p.kseq_ndrafts;
    io.kseq_pos = reinterpret_cast<int32_t *>(p.ws + p.lay.kseq_pos);
    FinalOut fo;
    fo.sel = reinterpret_cast<Selection *>(p.ws + p.lay.sel);
    fo.partial = reinterpret_cast<SegPartial *>(p.ws + p.lay.partial);
    fo.counter = reinterpret_cast<int32_t *>(p.ws + p.lay.counter);
    fo.res_norm = reinterpret_cast<double *>(p.ws + p.lay.res_norm);
    fo.u_final = reinterpret_cast<double *>(p.ws + p.lay.u_final);
    fo.margin = reinterpret_cast<double *>(p.ws + p.lay.margin);
    fo.fallback = reinterpret_cast<int32_t *>(p.ws + p.lay.fallback);
    fo.carry = reinterpret_cast<double *>(p.ws + p.lay.carry);
    fo.mcount = reinterpret_cast<int32_t *>(p.ws + p.lay.mcount);
    fo.state_carry = p.state_carry; fo.state_count = p.state_count;
    const int KL = p.K * p.L;
    const size_t lds = sizeof(double) * (6 * KL + p.K) + sizeof(int) * KL + ((static_cast<size_t>(p.K) * p.K + 7) & ~static_cast<size_t>(7));
#define SPECGBV_FINAL_LAUNCH(VEC, PEND)                                                                              \
    hipLaunchKernelGGL((k_final<T, VEC, PEND>), g, dim3(kSegThreads), lds, p.stream, target, draft, io, fo, p.V, p.K, \
                       p.L, p.c, p.lay.nseg, p.seed, p.offset)
    if (p.pend_levels > 0) { if (vec) SPECGBV_FINAL_LAUNCH(true, true); else SPECGBV_FINAL_LAUNCH(false, true); }
    else { if (vec) SPECGBV_FINAL_LAUNCH(true, false); else SPECGBV_FINAL_LAUNCH(false, false); }
#undef SPECGBV_FINAL_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decide_and_sample(const Problem &p)
{
    return p.dtype == 1 ? launch_final_typed<uint16_t>(p) : launch_final_typed<float>(p);
}

}  // namespace specgbv
