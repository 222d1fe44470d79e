// Schedule "split": two streaming passes over the logits.
//
//   k_row_stats : per row, log2 sum_x 2^(c z[x]) and the token's scaled logit
//                 (soft-max statistics of the distributions Algorithm 1 takes as input)
//   k_ot_sum    : per row pair i = 1..L-1, the vocabulary sum of Eq. (hik) divided by
//                 q(x^i):  s_i = sum_x q_i[x] max(1 - p_i[x] / (nu_i q_i[x]), 0)^K
//
// With a pending distribution modification (Algorithm 2 applied on the fly) a third kernel
// runs between the two:
//   k_pend_norm : per modified row, the block ratio mu Algorithm 2 uses there, the normaliser
//                 N = sum_x q[x] max(1 - p[x] / (mu q[x]), 0)^K of q_new, and the drafted
//                 token's factor,
// and k_ot_sum evaluates its sum against q_new = q t^K / N formed per entry (one pass of k_pend_norm per
// pending level; a level's rows are shared among workgroups when it has few of them left).
//
// Small batches, where a workgroup per row would leave most of the chip idle, use k_row_stats_parts and
// k_ot_sum_parts instead: every row is cut into
// parts, combined in part order by the consumers.
//
// Any V and any alignment is accepted (rows whose byte length is not a multiple of 16
// take the scalar-load path).  This schedule reads every row pair twice; it is the
// general fallback and the reference schedule for the on-chip "chain" kernel.
#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kStatThreads = 512;
constexpr int kMaxRows = 64;         // rows of a draft (L <= 62)
static_assert(kRowParts <= kPendParts, "the partial Eq. (hik) sums use the level passes' buffer");

// What the level passes need before they start (pending modifications only): per level l and prefix b the
// number of rows the level modifies in the prefixes before b, K * sum_{b' < b} clamp(count[l][b'], 0, L), with the
// level's total at position batch.  One workgroup per level.
__device__ __forceinline__ void pend_offsets(const int32_t *count_l, int K, int L, int batch, int32_t *off_l)
{
    __shared__ double sh_scan[kStatThreads / kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wid = tid / kWave;
    const int chunk = (batch + kStatThreads - 1) / kStatThreads;
    const int b0 = tid * chunk, b1 = b0 + chunk < batch ? b0 + chunk : batch;
    double mine = 0.0;                                 // small integers: exact in float64
    for (int b = b0; b < b1; ++b) {
        const int cnt = count_l[b];
        mine += static_cast<double>(K) * static_cast<double>(cnt < 0 ? 0 : (cnt > L ? L : cnt));
    }
    const double incl = wave_inclusive_sum(mine);
    if (lane == kWave - 1) sh_scan[wid] = incl;
    __syncthreads();
    double before = incl - mine;
    for (int w = 0; w < wid; ++w) before += sh_scan[w];
    for (int b = b0; b < b1; ++b) {
        off_l[b] = static_cast<int32_t>(before);
        const int cnt = count_l[b];
        before += static_cast<double>(K) * static_cast<double>(cnt < 0 ? 0 : (cnt > L ? L : cnt));
    }
    if (tid == kStatThreads - 1) off_l[batch] = static_cast<int32_t>(before);     // the last thread's end is the total
}

// grid (row pairs + pending levels, 2): blocks (pair, 0 / 1) reduce the target / draft row of the pair; with
// pending modifications blocks (pairs + l, 0) compute level l's offsets (pend_offsets) and the row blocks clear
// the arrival counters of the level passes.
template <typename T, bool VEC>
__global__ void __launch_bounds__(kStatThreads)
k_row_stats(const T *__restrict__ target, const T *__restrict__ draft,
            const int32_t *__restrict__ tokens, int K, int L, int V, float c,
            RowStat *__restrict__ stats, int32_t *__restrict__ final_counter, long long n_rows, int batch,
            const int32_t *__restrict__ pend_count, int32_t *__restrict__ pend_off, int32_t *__restrict__ pend_cnt,
            double c_rel)
{
    __shared__ double sh_d[kStatThreads / kWave];
    __shared__ float sh_f[kStatThreads / kWave];
    const long long pair = blockIdx.x;            // (b*K + k)*L + r
    const bool is_draft = blockIdx.y == 1;
    if (pair >= n_rows) {                         // uniform: one of the offset blocks
        const int level = static_cast<int>(pair - n_rows);
        if (!is_draft)
            pend_offsets(pend_count + static_cast<size_t>(level) * batch, K, L, batch,
                         pend_off + static_cast<size_t>(level) * (batch + 1));
        return;
    }
    const int r = static_cast<int>(pair % L);
    const long long bk = pair / L;
    if (threadIdx.x == 0 && !is_draft) {
        if (pair % (static_cast<long long>(K) * L) == 0)
            final_counter[pair / (static_cast<long long>(K) * L)] = 0;  // arrival counter of the final-token kernel
        if (pend_cnt) pend_cnt[pair] = 0;
    }
    const T *row = is_draft ? draft + (bk * L + r) * static_cast<long long>(V)
                            : target + (bk * (L + 1) + r) * static_cast<long long>(V);
    constexpr int PV = Elem<T>::kPerVec;
    const int tok_raw = token_index_queued(tokens, pair);
    RunningSum acc;                               // the drafted token is left out (leave_out)
    if (VEC) {
        const int nvec = V / PV;
        for (int i = threadIdx.x; i < nvec; i += kStatThreads) {
            const U4 v = load16_stream(row + static_cast<long long>(i) * PV);
            const int tok = token_index_used(tok_raw, V);
            float z[PV];
            Elem<T>::unpack(v, z);
            leave_out(z, i == tok / PV, tok % PV);
            acc.add(z, c);
        }
    } else {
        for (int x = threadIdx.x; x < V; x += kStatThreads) {
            float z[1] = {Elem<T>::scalar(row + x)};
            leave_out(z, x == token_index_used(tok_raw, V), 0);
            acc.add(z, c);
        }
    }
    const int tok = token_index_used(tok_raw, V);
    const float M = block_max(acc.m2, sh_f);
    const double part = static_cast<double>(acc.Z) * exp2(static_cast<double>(acc.m2) - static_cast<double>(M));
    const double total = block_sum(acc.Z > 0.0f ? part : 0.0, sh_d);
    if (threadIdx.x == 0) {
        const double tok2_raw = static_cast<double>(Elem<T>::scalar(row + tok)) * static_cast<double>(c);
        const RefSum all = with_token(static_cast<double>(M), total, tok2_raw);
        const double lse2 = all.ref + log2(all.Z);
        const double tok2 = token_scaled(tok2_raw, lse2, c_rel);
        if (is_draft) { stats[pair].lse2_p = lse2; stats[pair].tok2_p = tok2; }
        else { stats[pair].lse2_q = lse2; stats[pair].tok2_q = tok2; }
    }
}

// ---- small batches: rows shared among workgroups
//
// With few rows a workgroup per row leaves most of the chip idle and every workgroup pays the latency of
// streaming a whole row alone (16 - 21 us per kernel at one prefix, whatever the bandwidth).  Each row (pair) is
// then cut into P parts: k_row_stats_parts leaves partial statistics with integral reference exponents,
// k_ot_sum_parts combines the ones each of its workgroups needs (and stores the RowStat entries) and leaves P
// partial sums per row, which the final-token kernel adds up in part order.  No workgroup waits for another one.

// grid (row pairs * P, 2): block (pair * P + part, 0 / 1) reduces part `part` of the target / draft row of the pair
template <typename T, bool VEC>
__global__ void __launch_bounds__(kStatThreads)
k_row_stats_parts(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens, int L,
                  int V, float c, int P, Row0Part *__restrict__ parts)
{
    __shared__ double sh_d[kStatThreads / kWave];
    __shared__ float sh_f[kStatThreads / kWave];
    const long long pair = blockIdx.x / P;        // (b*K + k)*L + r
    const int part = static_cast<int>(blockIdx.x % P);
    const int r = static_cast<int>(pair % L);
    const long long bk = pair / L;
    const bool is_draft = blockIdx.y == 1;
    const T *row = is_draft ? draft + (bk * L + r) * static_cast<long long>(V)
                            : target + (bk * (L + 1) + r) * static_cast<long long>(V);
    constexpr int PV = Elem<T>::kPerVec;
    const int units = VEC ? V / PV : V;
    const int per = (units + P - 1) / P;
    const int lo = part * per, hi = lo + per < units ? lo + per : units;
    const int tok_raw = token_index_queued(tokens, pair);
    RunningSum acc;                               // the drafted token is left out (leave_out)
    if (VEC) {
        int i = lo + static_cast<int>(threadIdx.x);
        for (; i + kStatThreads < hi; i += 2 * kStatThreads) {            // two loads in flight per thread
            const U4 a = load16_stream(row + static_cast<long long>(i) * PV);
            const U4 b2 = load16_stream(row + static_cast<long long>(i + kStatThreads) * PV);
            const int tk = token_index_used(tok_raw, V);
            float z[PV];
            Elem<T>::unpack(a, z); leave_out(z, i == tk / PV, tk % PV); acc.add(z, c);
            Elem<T>::unpack(b2, z); leave_out(z, i + kStatThreads == tk / PV, tk % PV); acc.add(z, c);
        }
        if (i < hi) {
            const U4 a = load16_stream(row + static_cast<long long>(i) * PV);
            const int tk = token_index_used(tok_raw, V);
            float z[PV];
            Elem<T>::unpack(a, z);
            leave_out(z, i == tk / PV, tk % PV);
            acc.add(z, c);
        }
    } else {
        for (int x = lo + static_cast<int>(threadIdx.x); x < hi; x += kStatThreads) {
            float z[1] = {Elem<T>::scalar(row + x)};
            leave_out(z, x == token_index_used(tok_raw, V), 0);
            acc.add(z, c);
        }
    }
    const int tok = token_index_used(tok_raw, V);
    const int tok_unit = VEC ? tok / PV : tok;
    const float M = block_max(acc.m2, sh_f);
    const double mine = static_cast<double>(acc.Z) * exp2(static_cast<double>(acc.m2) - static_cast<double>(M));
    const double total = block_sum(acc.Z > 0.0f ? mine : 0.0, sh_d);
    if (threadIdx.x == 0) {
        // the part that holds the drafted token adds its weight here, in float64
        const bool mine_tok = tok_unit >= lo && tok_unit < hi;
        const double tok2_raw = mine_tok ? static_cast<double>(Elem<T>::scalar(row + tok)) * static_cast<double>(c)
                                         : -static_cast<double>(__builtin_inff());
        const RefSum all = with_token(static_cast<double>(M), total, tok2_raw);
        Row0Part out;
        out.ref = floor(all.ref);
        out.Z = all.Z * exp2(all.ref - out.ref);
        parts[(pair * 2 + (is_draft ? 1 : 0)) * kRowParts + part] = out;
    }
}

// log2 sum_x 2^(c z[x]) of a row from its parts' sums (combined in part order: the same bits wherever it is done)
__device__ __forceinline__ double lse2_from_parts(const Row0Part *pp, int P)
{
    double ref = -1.0e300;
    for (int q = 0; q < P; ++q)
        if (pp[q].Z > 0.0 && pp[q].ref > ref) ref = pp[q].ref;
    double Z = 0.0;
    for (int q = 0; q < P; ++q) {
        const double d = pp[q].ref - ref;                     // an integer <= 0
        if (pp[q].Z > 0.0 && d > -2000.0) Z += ldexp(pp[q].Z, static_cast<int>(d));
    }
    return ref + log2(Z);
}

// The drafted token's term of a row's Eq. (hik) sum in float64 in place of the sweep's float32 value (see
// token_term): called by one thread with the sum `total` (relative to 2^shift_q) of the entries [lo, hi) of the
// row; returns total with the term exchanged if the token (*token) is among them, or total itself where the term
// needs no second look (decided from the row's statistics: the token is not even fetched then).
template <typename T>
__device__ __forceinline__ double with_token_term(double total, const RowStat &st, double log2nu, const T *rq, const T *rp,
                                                  const int32_t *token, int V, int lo, int hi, float c, float shift_q,
                                                  const RatioConst &rc, int K)
{
    const double log2q = st.tok2_q - st.lse2_q, log2r = (st.tok2_p - st.lse2_p) - log2q - log2nu;
    if (!(fabs(1.0 - exp2_small(log2r)) < static_cast<double>(kTokenTermBelow))) return total;
    int tok = *token;
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    if (tok < lo || tok >= hi) return total;
    const float zq[1] = {Elem<T>::scalar(rq + tok)}, zp[1] = {Elem<T>::scalar(rp + tok)};
    float wq[1], w[1];
    ot_weights(zq, zp, c, shift_q, rc, K, wq, w);            // the same operations as in the sweep: the same bits
    return (total - static_cast<double>(w[0])) + token_term(log2q, log2r, K) * exp2_small(st.lse2_q - static_cast<double>(shift_q));
}

// grid rows * P, rows = batch * K * (L - 1): block row * P + part sums part `part` of the Eq. (hik) terms of row
// pair i = 1 .. L-1 of a draft (PEND: against the row as the pending levels leave it, exactly as k_ot_sum does).
// With stat_P > 1 the statistics of the draft's rows 0 .. i are still in parts
// (k_row_stats_parts): every workgroup combines the ones it needs, and part 0 stores the RowStat entry of its
// row (the workgroup of row 1 also that of row 0, and clears the arrival counter of the final-token kernel).
template <typename T, bool VEC, bool PEND>
__global__ void __launch_bounds__(kStatThreads)
k_ot_sum_parts(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens, int K, int L,
               int V, float c, int P, const Row0Part *__restrict__ stat_parts, int stat_P, RowStat *stats,
               int32_t *__restrict__ final_counter, double *__restrict__ s_part, double *__restrict__ e_part,
               const PendRow *__restrict__ pend, long long n_rows, int nlev, double c_rel)
{
    __shared__ double sh_d[kStatThreads / kWave];
    __shared__ PendTable sh_tab;                  // PEND: the levels that modify this row
    __shared__ PendRow sh_pr[kMaxPend];
    __shared__ double sh_sumN;
    __shared__ double sh_lse[2 * kMaxRows], sh_tok[2 * kMaxRows];
    const long long idx = blockIdx.x / P;         // bk*(L-1) + (i-1)
    const int part = static_cast<int>(blockIdx.x % P);
    const int i = static_cast<int>(idx % (L - 1)) + 1;
    const long long bk = idx / (L - 1);
    const long long pair = bk * L + i;
    RowStat st;
    double log2nu = 0.0;
    if (stat_P > 1) {
        for (int t = threadIdx.x; t < 2 * (i + 1); t += kStatThreads) {
            const int j = t >> 1, m = t & 1;
            const long long pj = bk * L + j;
            sh_lse[t] = lse2_from_parts(stat_parts + (pj * 2 + m) * kRowParts, stat_P);
            int tok = tokens[pj];
            tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
            const T *row = m ? draft + pj * static_cast<long long>(V) : target + (bk * (L + 1) + j) * static_cast<long long>(V);
            sh_tok[t] = token_scaled(static_cast<double>(Elem<T>::scalar(row + tok)) * static_cast<double>(c), sh_lse[t], c_rel);
        }
        __syncthreads();
        st.lse2_q = sh_lse[2 * i]; st.lse2_p = sh_lse[2 * i + 1];
        st.tok2_q = sh_tok[2 * i]; st.tok2_p = sh_tok[2 * i + 1];
        for (int j = 0; j < i; ++j) log2nu += (sh_tok[2 * j] - sh_lse[2 * j]) - (sh_tok[2 * j + 1] - sh_lse[2 * j + 1]);
        if (part == 0 && threadIdx.x == 0) {
            stats[pair] = st;
            if (i == 1) {
                RowStat s0;
                s0.lse2_q = sh_lse[0]; s0.lse2_p = sh_lse[1]; s0.tok2_q = sh_tok[0]; s0.tok2_p = sh_tok[1];
                stats[bk * L] = s0;
                if (bk % K == 0) final_counter[bk / K] = 0;
            }
        }
    } else {
        st = stats[pair];
        if (!PEND)
            for (int j = 0; j < i; ++j) {
                const RowStat a = stats[bk * L + j];
                log2nu += (a.tok2_q - a.lse2_q) - (a.tok2_p - a.lse2_p);
            }
    }
    double sumN = 0.0;
    if (PEND) {                                   // as in k_ot_sum: the row as the pending levels leave it
        log2nu = pend_block_ratio(stats, pend, n_rows, nlev, bk * L, i, sh_d);
        if (static_cast<int>(threadIdx.x) < nlev) sh_pr[threadIdx.x] = pend[static_cast<long long>(threadIdx.x) * n_rows + pair];
        __syncthreads();
        if (threadIdx.x == 0) sh_sumN = pend_build_table(sh_pr, 1, nlev, 0, st.lse2_p - st.lse2_q, sh_tab);
        __syncthreads();
        sumN = sh_sumN;
    }
    const float shift_q = static_cast<float>(st.lse2_q);
    const T *rq = target + (bk * (L + 1) + i) * static_cast<long long>(V);
    const T *rp = draft + pair * static_cast<long long>(V);
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    const RatioConst rc(ratio_const(st.lse2_p, st.lse2_q, log2nu, c_rel) - sumN);
    const int units = VEC ? V / N : V;
    const int per = (units + P - 1) / P;
    const int lo = part * per, hi = lo + per < units ? lo + per : units;
    float acc = 0.0f;
    if (PEND && sh_tab.n > 0) {                   // uniform over the workgroup
        for_each_pair_range<T, VEC, kStatThreads>(rq, rp, lo, hi, [&](int, const float (&zq)[N], const float (&zp)[N]) {
            float wq[N], w[N];
            pending_weights(zq, zp, c, shift_q, sh_tab, rc, K, wq, w);
#pragma unroll
            for (int j = 0; j < N; ++j) acc += w[j];
        });
    } else {
        for_each_pair_range<T, VEC, kStatThreads>(rq, rp, lo, hi, [&](int, const float (&zq)[N], const float (&zp)[N]) {
            float wq[N], w[N];
            ot_weights(zq, zp, c, shift_q, rc, K, wq, w);
#pragma unroll
            for (int j = 0; j < N; ++j) acc += w[j];
        });
    }
    double total = block_sum(static_cast<double>(acc), sh_d);
    if (threadIdx.x == 0 && !(PEND && sh_tab.n > 0))
        total = with_token_term<T>(total, st, log2nu, rq, rp, tokens + pair, V, lo * N, hi * N, c, shift_q, rc, K);
    // (whether the row's s and g nearly cancel, so that Eq. (hik) needs nu^2 (s - g) summed term by term, only the sum
    // over all parts can tell: the final-token kernel looks at it)
    if (threadIdx.x == 0) s_part[pair * kPendParts + part] = total * exp2(static_cast<double>(shift_q) - st.lse2_q - sumN);
    // (the final-token kernel looks at the complete sums itself and takes E where a row needs it: its parts start as
    // "not there yet")
    if (part == 0 && threadIdx.x < kPendParts) e_part[pair * kPendParts + threadIdx.x] = -1.0;
}

// One level of pending modification (the levels below it are done: their PendRow entries are read).
// grid.x >= batch * K * L.  Workgroup w first writes the empty entry of row pair w (if there is one) if the level
// leaves that row alone.  Then it takes a unit of work: the T rows the level modifies are enumerated prefix by prefix (off[b] rows
// before prefix b; within a prefix row index slowest) and each is shared among P = min(grid / T, kPendParts)
// workgroups, so that a level with few rows left still occupies the chip (one workgroup streaming a whole row
// pair with several levels of arithmetic per entry takes 100 - 200 us).  Unit u = blockIdx.x < T * P is part
// u % P of row u / P; the parts' sums meet in the workspace (device-scope relaxed atomic accesses) and the
// workgroup that arrives last at the row's counter finishes the row.  No workgroup waits for another one.
template <typename T, bool VEC>
__global__ void __launch_bounds__(kStatThreads)
k_pend_norm(const T *__restrict__ target, const T *__restrict__ draft, int K, int L, int V, float c,
            const double *__restrict__ carry_l, const int32_t *__restrict__ count_l,
            const RowStat *__restrict__ stats, PendRow *pend, long long n_rows, int level,
            const int32_t *__restrict__ off, int batch, double *part_buf, int32_t *arrive)
{
    __shared__ double sh_d[kStatThreads / kWave];
    __shared__ PendTable sh_tab;
    __shared__ PendRow sh_pr[kMaxPend];           // the levels below, at this row
    __shared__ double sh_log2mu, sh_sumN;
    __shared__ int sh_b, sh_last;
    PendRow out;
    out.log2mu = 0.0; out.log2N = 0.0; out.tokadj = 0.0; out.flag = 0; out.pad = 0;
    {
        const long long pair0 = blockIdx.x;
        const int r0 = static_cast<int>(pair0 % L);
        if (threadIdx.x == 0 && pair0 < n_rows && r0 >= count_l[(pair0 / L) / K]) pend[level * n_rows + pair0] = out;
    }
    const int T_live = off[batch];
    if (T_live <= 0) return;                      // uniform over the grid
    int P = static_cast<int>(gridDim.x / static_cast<unsigned>(T_live));   // >= 1: the modified rows are among the grid's rows
    P = P > kPendParts ? kPendParts : P;
    if (static_cast<long long>(blockIdx.x) >= static_cast<long long>(T_live) * P) return;
    const int item = static_cast<int>(blockIdx.x) / P, part = static_cast<int>(blockIdx.x) % P;
    for (int base = 0; base < batch; base += kStatThreads) {
        const int bb = base + static_cast<int>(threadIdx.x);
        if (bb < batch && off[bb] <= item && item < off[bb + 1]) sh_b = bb;          // exactly one thread
    }
    __syncthreads();
    const int b = sh_b;
    const int j = item - off[b];
    const int r = j / K;
    const long long bk = static_cast<long long>(b) * K + j % K;
    const long long pair = bk * L + r;            // (b*K + k)*L + r
    const RowStat st = stats[pair];
    // block ratio in front of row r: the carried one continued along the drafted tokens with the
    // distribution this level modifies (the target rows as modified by the levels below)
    const double ahead = pend_block_ratio(stats, pend, n_rows, level, bk * L, r, sh_d);
    if (static_cast<int>(threadIdx.x) < level) sh_pr[threadIdx.x] = pend[static_cast<long long>(threadIdx.x) * n_rows + pair];
    __syncthreads();
    if (threadIdx.x == 0) {
        sh_log2mu = carry_l[b] * 1.44269504088896340736 + ahead;
        sh_sumN = pend_build_table(sh_pr, 1, level, 0, st.lse2_p - st.lse2_q, sh_tab);
    }
    __syncthreads();
    const double log2mu = sh_log2mu, sumN = sh_sumN;
    const float shift_q = static_cast<float>(st.lse2_q);
    const RatioConst rc(st.lse2_p - st.lse2_q + log2mu - sumN);
    const T *rq = target + (bk * (L + 1) + r) * static_cast<long long>(V);
    const T *rp = draft + pair * static_cast<long long>(V);
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    const int units = VEC ? V / N : V;
    const int per = (units + P - 1) / P;
    const int lo = part * per, hi = lo + per < units ? lo + per : units;
    float acc = 0.0f;
    if (sh_tab.n == 0) {
        for_each_pair_range<T, VEC, kStatThreads>(rq, rp, lo, hi, [&](int, const float (&zq)[N], const float (&zp)[N]) {
            float wq[N], w[N];
            ot_weights(zq, zp, c, shift_q, rc, K, wq, w);
#pragma unroll
            for (int jj = 0; jj < N; ++jj) acc += w[jj];
        });
    } else {
        for_each_pair_range<T, VEC, kStatThreads>(rq, rp, lo, hi, [&](int, const float (&zq)[N], const float (&zp)[N]) {
            float wq[N], w[N];
            pending_weights(zq, zp, c, shift_q, sh_tab, rc, K, wq, w);
#pragma unroll
            for (int jj = 0; jj < N; ++jj) acc += w[jj];
        });
    }
    double S = block_sum(static_cast<double>(acc), sh_d);                 // relative to 2^shift_q
    if (P > 1) {
        // the store is a device-scope access; the workgroup-scope release fence waits until it has completed,
        // so the counter update that follows (same thread) cannot be seen before it
        if (threadIdx.x == 0) {
            __hip_atomic_store(reinterpret_cast<unsigned long long *>(part_buf + pair * kPendParts + part),
                               static_cast<unsigned long long>(__double_as_longlong(S)), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            const int arrived = __hip_atomic_fetch_add(&arrive[pair], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh_last = arrived == P - 1;
        }
        __syncthreads();
        if (!sh_last) return;
        if (threadIdx.x == 0) {
            S = 0.0;
            for (int q = 0; q < P; ++q)                                   // in part order: the same bits whoever finishes
                S += __longlong_as_double(static_cast<long long>(__hip_atomic_load(
                    reinterpret_cast<const unsigned long long *>(part_buf + pair * kPendParts + q), __ATOMIC_RELAXED,
                    __HIP_MEMORY_SCOPE_AGENT)));
            __hip_atomic_store(&arrive[pair], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next level's pass
        }
    }
    if (threadIdx.x == 0) {
        const double W = S * exp2(static_cast<double>(shift_q) - st.lse2_q - sumN);   // mass of q^(level) t^K
        out.log2mu = log2mu;
        if (W > 0.0) {                            // otherwise every weight is zero and the row stays q^(level)
            out.flag = 1;
            out.log2N = log2(W);
            const double tq_eff = (st.tok2_q - st.lse2_q) + pend_token_adjust(sh_pr, 1, level, 0);
            const double ratio = exp2((st.tok2_p - st.lse2_p) - tq_eff - log2mu);
            const double t = 1.0 - ratio;
            out.tokadj = t > 0.0 ? static_cast<double>(K) * log2(t) : -INFINITY;
        }
        pend[level * n_rows + pair] = out;
    }
}

template <typename T, bool VEC, bool PEND>
__global__ void __launch_bounds__(kStatThreads)
k_ot_sum(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens, int K, int L, int V,
         float c, const RowStat *__restrict__ stats, const PendRow *__restrict__ pend, long long n_rows, int nlev,
         double *__restrict__ s_out, double *__restrict__ e_out, double *__restrict__ e_part, double c_rel)
{
    __shared__ double sh_d[kStatThreads / kWave];
    __shared__ PendTable sh_tab;
    __shared__ PendRow sh_pr[kMaxPend];           // the levels, at this row
    __shared__ double sh_sumN;
    const long long idx = blockIdx.x;             // bk*(L-1) + (i-1)
    const int i = static_cast<int>(idx % (L - 1)) + 1;
    const long long bk = idx / (L - 1);
    const RowStat st = stats[bk * L + i];
    // block likelihood ratio of the length-i block, from the rows before row i (their token
    // probabilities under the modified rows where levels are pending)
    double log2nu = 0.0, sumN = 0.0;
    if (PEND) {
        log2nu = pend_block_ratio(stats, pend, n_rows, nlev, bk * L, i, sh_d);
        if (static_cast<int>(threadIdx.x) < nlev) sh_pr[threadIdx.x] = pend[static_cast<long long>(threadIdx.x) * n_rows + bk * L + i];
        __syncthreads();
        if (threadIdx.x == 0) sh_sumN = pend_build_table(sh_pr, 1, nlev, 0, st.lse2_p - st.lse2_q, sh_tab);
        __syncthreads();
        sumN = sh_sumN;
    } else {
        for (int j = 0; j < i; ++j) {
            const RowStat a = stats[bk * L + j];
            log2nu += (a.tok2_q - a.lse2_q) - (a.tok2_p - a.lse2_p);
        }
    }
    const float shift_q = static_cast<float>(st.lse2_q);
    const T *rq = target + (bk * (L + 1) + i) * static_cast<long long>(V);
    const T *rp = draft + (bk * L + i) * static_cast<long long>(V);
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    const RatioConst rc(ratio_const(st.lse2_p, st.lse2_q, log2nu, c_rel) - sumN);
    float acc = 0.0f;
    if (PEND && sh_tab.n > 0) {                   // uniform over the workgroup
        for_each_pair<T, VEC, kStatThreads>(rq, rp, V, [&](int, const float (&zq)[N], const float (&zp)[N]) {
            float wq[N], w[N];
            pending_weights(zq, zp, c, shift_q, sh_tab, rc, K, wq, w);
#pragma unroll
            for (int j = 0; j < N; ++j) acc += w[j];
        });
    } else {
        for_each_pair<T, VEC, kStatThreads>(rq, rp, V, [&](int, const float (&zq)[N], const float (&zp)[N]) {
            float wq[N], w[N];
            ot_weights(zq, zp, c, shift_q, rc, K, wq, w);
#pragma unroll
            for (int j = 0; j < N; ++j) acc += w[j];
        });
    }
    double total = block_sum(static_cast<double>(acc), sh_d);
    if (threadIdx.x == 0 && !(PEND && sh_tab.n > 0))
        total = with_token_term<T>(total, st, log2nu, rq, rp, tokens + (bk * L + i), V, 0, V, c, shift_q, rc, K);
    const double s_val = total * exp2(static_cast<double>(shift_q) - st.lse2_q - sumN);
    // where s and g = (1 - 1/nu)^K nearly cancel, Eq. (hik) needs nu^2 (s - g) summed term by term (rare: peaked
    // rows, large block ratios): the final-token kernel finds those rows and its workgroups sum E together (the
    // parts start as "not there yet")
    const double e_val = -1.0;
    if (threadIdx.x < kPendParts) e_part[(bk * L + i) * kPendParts + threadIdx.x] = -1.0;
    if (threadIdx.x == 0) { s_out[bk * L + i] = s_val; e_out[bk * L + i] = e_val; }
}

int compute_units()
{
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        cached[dev] = (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
    }
    return cached[dev];
}

// Parts a row is cut into so that about four workgroups per compute unit are launched (1: one workgroup per row).
int row_parts(long long workgroups_per_row_unit, int V)
{
    if (V < 8192 || workgroups_per_row_unit < 1) return 1;         // short rows: nothing to share
    const long long want = 4LL * compute_units() / workgroups_per_row_unit;
    // below four parts the partial sums' extra steps cost what the sharing gains (measured)
    return static_cast<int>(want < 4 ? 1 : (want > kRowParts ? kRowParts : want));
}

template <typename T>
hipError_t launch_typed(const Problem &p)
{
    const T *target = static_cast<const T *>(p.target);
    const T *draft = static_cast<const T *>(p.draft);
    RowStat *stats = reinterpret_cast<RowStat *>(p.ws + p.lay.stats);
    double *s = reinterpret_cast<double *>(p.ws + p.lay.s);
    int32_t *counter = reinterpret_cast<int32_t *>(p.ws + p.lay.counter);
    const long long pairs = static_cast<long long>(p.batch) * p.K * p.L;
    const bool vec = (p.V % Elem<T>::kPerVec) == 0 &&
                     (reinterpret_cast<uintptr_t>(p.target) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(p.draft) % 16 == 0);
    int32_t *pend_off = reinterpret_cast<int32_t *>(p.ws + p.lay.pend_off);
    int32_t *pend_cnt = p.pend_levels > 0 ? reinterpret_cast<int32_t *>(p.ws + p.lay.pend_cnt) : nullptr;
    double *pend_part = reinterpret_cast<double *>(p.ws + p.lay.pend_part);
    // rows shared among workgroups (small batches); the sums' kernel then finishes the statistics, so L >= 2
    const int stat_parts = (p.pend_levels > 0 || p.s_parts < 2) ? 1 : row_parts(2 * pairs, p.V);
    Row0Part *stat_part = reinterpret_cast<Row0Part *>(p.ws + p.lay.stat_part);
    if (stat_parts > 1) {
        const dim3 gs(static_cast<unsigned>(pairs * stat_parts), 2);
        if (vec)
            hipLaunchKernelGGL((k_row_stats_parts<T, true>), gs, dim3(kStatThreads), 0, p.stream, target, draft, p.tokens,
                               p.L, p.V, p.c, stat_parts, stat_part);
        else
            hipLaunchKernelGGL((k_row_stats_parts<T, false>), gs, dim3(kStatThreads), 0, p.stream, target, draft, p.tokens,
                               p.L, p.V, p.c, stat_parts, stat_part);
    } else {
        const dim3 g1(static_cast<unsigned>(pairs + p.pend_levels), 2);
        if (vec)
            hipLaunchKernelGGL((k_row_stats<T, true>), g1, dim3(kStatThreads), 0, p.stream, target, draft,
                               p.tokens, p.K, p.L, p.V, p.c, stats, counter, pairs, p.batch, p.pend_count, pend_off, pend_cnt, p.c_rel);
        else
            hipLaunchKernelGGL((k_row_stats<T, false>), g1, dim3(kStatThreads), 0, p.stream, target, draft,
                               p.tokens, p.K, p.L, p.V, p.c, stats, counter, pairs, p.batch, p.pend_count, pend_off, pend_cnt, p.c_rel);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    PendRow *pend = reinterpret_cast<PendRow *>(p.ws + p.lay.pend);
    for (int level = 0; level < p.pend_levels; ++level) {
        // one workgroup per row pair, but at least about four per compute unit, so that a small batch's rows can be shared
        const long long min_grid = 4LL * compute_units();
        const dim3 gp(static_cast<unsigned>(pairs > min_grid ? pairs : min_grid));
        const double *carry_l = p.pend_carry + static_cast<size_t>(level) * p.batch;
        const int32_t *count_l = p.pend_count + static_cast<size_t>(level) * p.batch;
        const int32_t *off_l = pend_off + static_cast<size_t>(level) * (p.batch + 1);
        if (vec)
            hipLaunchKernelGGL((k_pend_norm<T, true>), gp, dim3(kStatThreads), 0, p.stream, target, draft, p.K, p.L,
                               p.V, p.c, carry_l, count_l, stats, pend, pairs, level, off_l, p.batch, pend_part, pend_cnt);
        else
            hipLaunchKernelGGL((k_pend_norm<T, false>), gp, dim3(kStatThreads), 0, p.stream, target, draft, p.K, p.L,
                               p.V, p.c, carry_l, count_l, stats, pend, pairs, level, off_l, p.batch, pend_part, pend_cnt);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (p.L < 2) return hipSuccess;
    const long long rows = static_cast<long long>(p.batch) * p.K * (p.L - 1);
    if (p.s_parts > 1) {                            // small batch: partial sums, added up by the final-token kernel
        const dim3 gq(static_cast<unsigned>(rows * p.s_parts));
#define SPECGBV_OTP_LAUNCH(VEC, PEND)                                                                                 \
    do {                                                                                                              \
        hipLaunchKernelGGL((k_ot_sum_parts<T, VEC, PEND>), gq, dim3(kStatThreads), 0, p.stream, target, draft, p.tokens, \
                           p.K, p.L, p.V, p.c, p.s_parts, stat_part, stat_parts, stats, counter, pend_part,            \
                           reinterpret_cast<double *>(p.ws + p.lay.excess_part), pend, pairs, p.pend_levels, p.c_rel);  \
    } while (0)
        if (p.pend_levels > 0) { if (vec) SPECGBV_OTP_LAUNCH(true, true); else SPECGBV_OTP_LAUNCH(false, true); }
        else { if (vec) SPECGBV_OTP_LAUNCH(true, false); else SPECGBV_OTP_LAUNCH(false, false); }
#undef SPECGBV_OTP_LAUNCH
        return hipGetLastError();
    }
    const dim3 g2(static_cast<unsigned>(rows));
#define SPECGBV_OT_LAUNCH(VEC, PEND)                                                                           \
    hipLaunchKernelGGL((k_ot_sum<T, VEC, PEND>), g2, dim3(kStatThreads), 0, p.stream, target, draft, p.tokens, p.K, p.L, \
                       p.V, p.c, stats, pend, pairs, p.pend_levels, s, reinterpret_cast<double *>(p.ws + p.lay.excess),        \
                       reinterpret_cast<double *>(p.ws + p.lay.excess_part), p.c_rel)
    if (p.pend_levels > 0) { if (vec) SPECGBV_OT_LAUNCH(true, true); else SPECGBV_OT_LAUNCH(false, true); }
    else { if (vec) SPECGBV_OT_LAUNCH(true, false); else SPECGBV_OT_LAUNCH(false, false); }
#undef SPECGBV_OT_LAUNCH
    return hipGetLastError();
}

}  // namespace

int split_sum_parts(const Problem &p)
{
    if (p.L < 2) return 1;
    return row_parts(static_cast<long long>(p.batch) * p.K * (p.L - 1), p.V);
}

hipError_t launch_split_main(const Problem &p)
{
    return p.dtype == 1 ? launch_typed<uint16_t>(p) : launch_typed<float>(p);
}

}  // namespace specgbv
