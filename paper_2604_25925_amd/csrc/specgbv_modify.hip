// Distribution modification (Algorithm 2): the target distribution of the first rows of the
// next iteration.
//
// After an iteration accepted t^tau and drew the final token y, the first count = L - tau - 1
// rows of every new draft use
//     q_new[x] = w[x] / sum_x w[x],   w[x] = q_r[x] max(1 - p_r[x] / (nu q_r[x]), 0)^K
// (Algorithm 2 divided through by the joint probability of the conditioning block: the same
// per-token form as Eq. (pres)), with nu = [q(t^tau, y) / p(t^tau, y)] continued along the new
// draft's own tokens with the original target probabilities.
//
// Three streaming kernels, each with one workgroup per row (pair), so that any batch size
// fills the chip:
//   k_mod_stats : per row, log2 sum_x 2^(c z[x]) and the drafted token's scaled logit
//   k_mod_norm  : per modified row pair, nu (a prefix sum over the statistics of the rows
//                 before it) and the normaliser sum_x w[x]
//   k_mod_write : per row pair, natural-log probabilities in float32 (-inf where the
//                 probability is 0): ln q_new for modified rows, ln q otherwise, and ln p.
// An optional extra target row (the bonus row of the verification) is converted to
// log-probabilities as well, so that the whole output can be verified at temperature 1.
//
// Rows of up to kRowSlots * 512 sixteen-byte vectors take a shorter route: k_mod_row keeps a row in the registers of
// its workgroup between the statistics sweep and the store of its log-probabilities, so every row that no
// modification touches (all draft rows, the target rows from the prefix's count on, the bonus row) is read once;
// k_mod_norm and k_mod_write then run for the modified target rows only.
#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kModThreads = 512;

struct ModStat { double lse2, tok2; };       // base-2 log-normaliser, scaled logit of the row's token

// Workspace of one call: statistics of the target rows, of the draft rows, normalisers, flags.
struct ModLayout {
    size_t tstat, dstat, norm, fb, total;
};
__host__ __device__ inline size_t mod_align(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }
inline ModLayout mod_layout(int batch, int K, int M, int bonus)
{
    ModLayout l{};
    const size_t bk = static_cast<size_t>(batch) * K;
    size_t off = 0;
    l.tstat = off; off = mod_align(off + bk * (M + bonus) * sizeof(ModStat));
    l.dstat = off; off = mod_align(off + bk * M * sizeof(ModStat));
    l.norm = off; off = mod_align(off + bk * M * sizeof(double));
    l.fb = off; off = mod_align(off + bk * M * sizeof(int32_t));
    l.total = off;
    return l;
}

// grid.x = target rows followed by draft rows
template <typename T, bool VEC>
__global__ void __launch_bounds__(kModThreads)
k_mod_stats(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens,
            int M, int bonus, int V, float c, long long n_trows, ModStat *__restrict__ tstat,
            ModStat *__restrict__ dstat)
{
    __shared__ double sh_d[kModThreads / kWave];
    __shared__ float sh_f[kModThreads / kWave];
    const long long id = blockIdx.x;
    const bool is_draft = id >= n_trows;
    const long long row = is_draft ? id - n_trows : id;
    const T *z_row = (is_draft ? draft : target) + row * static_cast<long long>(V);
    const int rows_t = M + bonus;
    const int r = static_cast<int>(row % (is_draft ? M : rows_t));
    const long long bk = row / (is_draft ? M : rows_t);
    constexpr int PV = Elem<T>::kPerVec;
    RunningSum acc;
    if (VEC) {
        const int nvec = V / PV;
        int v = threadIdx.x;
        for (; v + kModThreads < nvec; v += 2 * kModThreads) {          // two loads in flight per thread
            const U4 a = load16_stream(z_row + static_cast<long long>(v) * PV);
            const U4 b = load16_stream(z_row + static_cast<long long>(v + kModThreads) * PV);
            float z[PV];
            Elem<T>::unpack(a, z); acc.add(z, c);
            Elem<T>::unpack(b, z); acc.add(z, c);
        }
        if (v < nvec) {
            float z[PV];
            Elem<T>::unpack(load16_stream(z_row + static_cast<long long>(v) * PV), z);
            acc.add(z, c);
        }
    } else {
        for (int x = threadIdx.x; x < V; x += kModThreads) {
            const float z[1] = {Elem<T>::scalar(z_row + x)};
            acc.add(z, c);
        }
    }
    const float Mx = block_max(acc.m2, sh_f);
    const double total = block_sum(static_cast<double>(acc.Z * exp2_fast(acc.m2 - Mx)), sh_d);
    if (threadIdx.x == 0) {
        ModStat st;
        st.lse2 = static_cast<double>(Mx) + log2(total);
        st.tok2 = 0.0;
        if (r < M) {                                   // the bonus row has no token
            int tok = tokens[bk * M + r];
            tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
            st.tok2 = static_cast<double>(Elem<T>::scalar(z_row + tok)) * static_cast<double>(c);
        }
        (is_draft ? dstat : tstat)[row] = st;
    }
}

constexpr int kRowSlots = 40;          // vectors per thread k_mod_row keeps: rows up to 163840 bfloat16 / 81920 float32 entries

// 8 (or 4) consecutive floats of an output row
template <int N>
__device__ __forceinline__ void store_vals(float *dst, const float (&v)[N])
{
    if (N % 4 == 0) {
#pragma unroll
        for (int j = 0; j < N; j += 4) *reinterpret_cast<float4 *>(dst + j) = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
    } else {
#pragma unroll
        for (int j = 0; j < N; ++j) dst[j] = v[j];
    }
}

// k_mod_stats for rows of at most kRowSlots * kModThreads vectors, with the row kept in registers: the workgroup
// then also writes the row's natural-log probabilities unless a modification is pending for it (target rows below
// the prefix's count: k_mod_norm and k_mod_write do those).  grid.x = target rows followed by draft rows; all of a
// thread's loads are issued before the first is used.
template <typename T>
__global__ void __launch_bounds__(kModThreads)
k_mod_row(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens, int K,
          int M, int bonus, int V, float c, long long n_trows, const int32_t *__restrict__ modify_count,
          ModStat *__restrict__ tstat, ModStat *__restrict__ dstat, float *__restrict__ out_logq,
          float *__restrict__ out_logp)
{
    constexpr float kLn2f = 0.693147180559945309417f;
    __shared__ double sh_d[kModThreads / kWave];
    __shared__ float sh_f[kModThreads / kWave];
    const long long id = blockIdx.x;
    const bool is_draft = id >= n_trows;
    const long long row = is_draft ? id - n_trows : id;
    const T *z_row = (is_draft ? draft : target) + row * static_cast<long long>(V);
    const int rows_t = M + bonus;
    const int r = static_cast<int>(row % (is_draft ? M : rows_t));
    const long long bk = row / (is_draft ? M : rows_t);
    constexpr int PV = Elem<T>::kPerVec;
    const int nvec = V / PV;                               // host: nvec <= kRowSlots * kModThreads
    const int tid = threadIdx.x;
    U4 v[kRowSlots];
#pragma unroll
    for (int j = 0; j < kRowSlots; ++j) {
        const int idx = j * kModThreads + tid;
        if (j * kModThreads < nvec)                        // (uniform: slots the row does not reach issue nothing)
            v[j] = load16_stream(z_row + static_cast<long long>(idx < nvec ? idx : nvec - 1) * PV);
        else
            v[j] = U4{0, 0, 0, 0};
    }
    RunningSum acc;
#pragma unroll
    for (int j = 0; j < kRowSlots; ++j) {
        if (j * kModThreads + tid < nvec) {
            float z[PV];
            Elem<T>::unpack(v[j], z);
            acc.add(z, c);
        }
    }
    const float Mx = block_max(acc.m2, sh_f);
    const double total = block_sum(static_cast<double>(acc.Z * exp2_fast(acc.m2 - Mx)), sh_d);
    const double lse2 = static_cast<double>(Mx) + log2(total);
    if (tid == 0) {
        ModStat st;
        st.lse2 = lse2;
        st.tok2 = 0.0;
        if (r < M) {                                       // the bonus row has no token
            int tok = tokens[bk * M + r];
            tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
            st.tok2 = static_cast<double>(Elem<T>::scalar(z_row + tok)) * static_cast<double>(c);
        }
        (is_draft ? dstat : tstat)[row] = st;
    }
    float *out = is_draft ? out_logp : out_logq;
    if (!is_draft && r < M && r < modify_count[bk / K]) out = nullptr;     // a modification is pending for this row
    if (!out) return;
    out += row * static_cast<long long>(V);
    // log2 prob[x] = fma(z, c, -h) - d with a float reference h and its float64 remainder d (as k_mod_write)
    const float h = static_cast<float>(lse2);
    const float dlt = static_cast<float>(lse2 - static_cast<double>(h));
#pragma unroll
    for (int j = 0; j < kRowSlots; ++j) {
        const int idx = j * kModThreads + tid;
        if (idx < nvec) {
            float z[PV], a[PV];
            Elem<T>::unpack(v[j], z);
#pragma unroll
            for (int e = 0; e < PV; ++e) a[e] = (fmaf(z[e], c, -h) - dlt) * kLn2f;
            store_vals(out + static_cast<long long>(idx) * PV, a);
        }
    }
}

// log2 of the block ratio in front of row r of draft bk: the carried ratio times the token
// ratios of rows 0..r-1 (original target probabilities).
__device__ __forceinline__ double mod_log2nu(const ModStat *tstat, const ModStat *dstat, long long bk, int rows_t,
                                             int M, int r, double carry_ln)
{
    double l = carry_ln * 1.44269504088896340736;
    for (int j = 0; j < r; ++j) {
        const ModStat a = tstat[bk * rows_t + j], b = dstat[bk * M + j];
        l += (a.tok2 - a.lse2) - (b.tok2 - b.lse2);
    }
    return l;
}

// grid.x = batch * K * M, row index slowest (the live workgroups, rows below the prefix's count, are then
// consecutive and spread over all dies whatever M is); row pairs with r >= count leave at once
template <typename T, bool VEC>
__global__ void __launch_bounds__(kModThreads)
k_mod_norm(const T *__restrict__ target, const T *__restrict__ draft, int K, int M, int bonus, int V, float c,
           const double *__restrict__ carry_log_nu, const int32_t *__restrict__ modify_count,
           const ModStat *__restrict__ tstat, const ModStat *__restrict__ dstat, double *__restrict__ norm,
           int32_t *__restrict__ fb_out)
{
    __shared__ double sh_d[kModThreads / kWave];
    const long long nbk = gridDim.x / M;
    const int r = static_cast<int>(blockIdx.x / nbk);
    const long long bk = blockIdx.x % nbk;
    const long long drow = bk * M + r;
    const int b = static_cast<int>(bk / K);
    const int rows_t = M + bonus;
    if (r >= modify_count[b]) {                       // uniform over the workgroup
        if (threadIdx.x == 0) { norm[drow] = 1.0; fb_out[drow] = 0; }
        return;
    }
    const ModStat sq = tstat[bk * rows_t + r], sp = dstat[drow];
    const float shift_q = static_cast<float>(sq.lse2);
    const RatioConst rc(sp.lse2 - sq.lse2 + mod_log2nu(tstat, dstat, bk, rows_t, M, r, carry_log_nu[b]));
    const T *rq = target + (bk * rows_t + r) * static_cast<long long>(V);
    const T *rp = draft + drow * static_cast<long long>(V);
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    float acc = 0.0f;
    for_each_pair<T, VEC, kModThreads>(rq, rp, V, [&](int, const float (&zq)[N], const float (&zp)[N]) {
        float wq[N], w[N];
        ot_weights(zq, zp, c, shift_q, rc, K, wq, w);
#pragma unroll
        for (int j = 0; j < N; ++j) acc += w[j];
    });
    const double S = block_sum(static_cast<double>(acc), sh_d);           // relative to 2^shift_q
    if (threadIdx.x == 0) {
        const double W = S * exp2(static_cast<double>(shift_q) - sq.lse2);
        const bool zero = !(W > 0.0);                // every weight is zero: the row stays q
        norm[drow] = zero ? 1.0 : W;
        fb_out[drow] = zero ? 1 : 0;
    }
}

// grid.x = batch * K * (M + bonus) target rows; plain_done: k_mod_row has written every row without a pending
// modification and all of ln p, so those workgroups leave at once
template <typename T, bool VEC>
__global__ void __launch_bounds__(kModThreads)
k_mod_write(const T *__restrict__ target, const T *__restrict__ draft, int K, int M, int bonus, int V, float c,
            const double *__restrict__ carry_log_nu, const int32_t *__restrict__ modify_count,
            const ModStat *__restrict__ tstat, const ModStat *__restrict__ dstat, const double *__restrict__ norm,
            const int32_t *__restrict__ fb_in, float *__restrict__ out_logq, float *__restrict__ out_logp, int plain_done)
{
    constexpr float kLn2f = 0.693147180559945309417f;
    const long long trow = blockIdx.x;
    const int rows_t = M + bonus;
    const int r = static_cast<int>(trow % rows_t);
    const long long bk = trow / rows_t;
    const int b = static_cast<int>(bk / K);
    const bool has_draft = r < M;
    const long long drow = bk * M + (has_draft ? r : M - 1);          // bonus row: any valid draft row, unused
    const ModStat sq = tstat[trow], sp = dstat[drow];
    // log2 q[x] = fma(z, c, -hq) - dq with a float reference hq and its float64 remainder dq
    const float hq = static_cast<float>(sq.lse2), hp = static_cast<float>(sp.lse2);
    const float dq = static_cast<float>(sq.lse2 - static_cast<double>(hq));
    const float dp = static_cast<float>(sp.lse2 - static_cast<double>(hp));
    if (plain_done && !(has_draft && r < modify_count[b])) return;     // (uniform over the workgroup)
    const bool modified = has_draft && r < modify_count[b] && fb_in[drow] == 0;
    const T *rq = target + trow * static_cast<long long>(V);
    const T *rp = has_draft ? draft + drow * static_cast<long long>(V) : rq;   // bonus row: no second stream
    float *oq = out_logq + trow * static_cast<long long>(V);
    float *op = (out_logp && has_draft && !plain_done) ? out_logp + drow * static_cast<long long>(V) : nullptr;
    constexpr int N = VEC ? Elem<T>::kPerVec : 1;
    if (modified) {
        // ln q_new = ln q + K ln t - ln W
        const RatioConst rc(sp.lse2 - sq.lse2 + mod_log2nu(tstat, dstat, bk, rows_t, M, r, carry_log_nu[b]));
        const float log2W = static_cast<float>(log2(norm[drow]) + sq.lse2 - static_cast<double>(hq));   // relative to 2^hq
        const float Kf = static_cast<float>(K);
        for_each_pair<T, VEC, kModThreads>(rq, rp, V, [&](int x, const float (&zq)[N], const float (&zp)[N]) {
            float a[N], bb[N];
#pragma unroll
            for (int j = 0; j < N; ++j) {
                a[j] = (fmaf(Kf, __log2f(rc.one_minus_ratio(zp[j] - zq[j], c)), fmaf(zq[j], c, -hq)) - log2W) * kLn2f;
                bb[j] = (fmaf(zp[j], c, -hp) - dp) * kLn2f;
            }
            store_vals(oq + x, a);
            if (op) store_vals(op + x, bb);
        });
    } else {
        for_each_pair<T, VEC, kModThreads>(rq, rp, V, [&](int x, const float (&zq)[N], const float (&zp)[N]) {
            float a[N], bb[N];
#pragma unroll
            for (int j = 0; j < N; ++j) {
                a[j] = (fmaf(zq[j], c, -hq) - dq) * kLn2f;
                bb[j] = (fmaf(zp[j], c, -hp) - dp) * kLn2f;
            }
            store_vals(oq + x, a);
            if (op) store_vals(op + x, bb);
        });
    }
}

template <typename T>
hipError_t launch_modify_typed(const void *target_v, const void *draft_v, const int32_t *tokens, int K, int M,
                               int bonus, int V, int batch, float c, const double *carry, const int32_t *count,
                               float *out_logq, float *out_logp, double *norm_out, int32_t *fallback_out,
                               char *ws, hipStream_t stream)
{
    const T *target = static_cast<const T *>(target_v), *draft = static_cast<const T *>(draft_v);
    const ModLayout lay = mod_layout(batch, K, M, bonus);
    ModStat *tstat = reinterpret_cast<ModStat *>(ws + lay.tstat), *dstat = reinterpret_cast<ModStat *>(ws + lay.dstat);
    double *norm = norm_out ? norm_out : reinterpret_cast<double *>(ws + lay.norm);
    int32_t *fb = fallback_out ? fallback_out : reinterpret_cast<int32_t *>(ws + lay.fb);
    const bool vec = (V % Elem<T>::kPerVec) == 0 && reinterpret_cast<uintptr_t>(target_v) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(draft_v) % 16 == 0 && reinterpret_cast<uintptr_t>(out_logq) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(out_logp) % 16 == 0;
    const long long bk = static_cast<long long>(batch) * K;
    const long long n_t = bk * (M + bonus), n_d = bk * M;
    const dim3 blk(kModThreads);
    // rows short enough to stay in a workgroup's registers are read once unless a modification is pending for them
    const bool rows_fit = vec && V / Elem<T>::kPerVec <= kRowSlots * kModThreads;
#define SPECGBV_MOD_LAUNCH(VEC)                                                                                   \
    do {                                                                                                          \
        if (rows_fit)                                                                                             \
            hipLaunchKernelGGL((k_mod_row<T>), dim3(static_cast<unsigned>(n_t + n_d)), blk, 0, stream, target,     \
                               draft, tokens, K, M, bonus, V, c, n_t, count, tstat, dstat, out_logq, out_logp);   \
        else                                                                                                      \
            hipLaunchKernelGGL((k_mod_stats<T, VEC>), dim3(static_cast<unsigned>(n_t + n_d)), blk, 0, stream,      \
                               target, draft, tokens, M, bonus, V, c, n_t, tstat, dstat);                         \
        hipLaunchKernelGGL((k_mod_norm<T, VEC>), dim3(static_cast<unsigned>(n_d)), blk, 0, stream, target, draft,  \
                           K, M, bonus, V, c, carry, count, tstat, dstat, norm, fb);                              \
        hipLaunchKernelGGL((k_mod_write<T, VEC>), dim3(static_cast<unsigned>(n_t)), blk, 0, stream, target, draft, \
                           K, M, bonus, V, c, carry, count, tstat, dstat, norm, fb, out_logq, out_logp,           \
                           rows_fit ? 1 : 0);                                                                     \
    } while (0)
    if (vec) SPECGBV_MOD_LAUNCH(true);
    else SPECGBV_MOD_LAUNCH(false);
#undef SPECGBV_MOD_LAUNCH
    return hipGetLastError();
}

// ---- advancing a pending modification's block ratio along the tokens an iteration emitted
//
// grid (M, batch).  Workgroup (j, b) handles emitted position j of prefix b: the token is draft
// f's j-th token for j < tau and the final token for j = tau; its log-ratio
// ln q_j[e] - ln p_j[e] under the rows the pending modification modifies goes to delta[b, j].
// Nothing is computed for prefixes whose modification expires with this iteration
// (count <= tau + 1) or that accepted a whole block.
template <typename T, bool VEC>
__global__ void __launch_bounds__(kModThreads)
k_carry_rows(const T *__restrict__ rows_q, const T *__restrict__ rows_p, const int32_t *__restrict__ tokens,
             const int32_t *__restrict__ accepted_len, const int32_t *__restrict__ accepted_idx,
             const int32_t *__restrict__ out_tokens, const int32_t *__restrict__ count, int K, int M, int rows_t,
             int V, float c, double *__restrict__ delta)
{
    __shared__ double sh_d[kModThreads / kWave];
    __shared__ float sh_f[kModThreads / kWave];
    const int j = blockIdx.x, b = blockIdx.y;
    const int tau = accepted_len[b];
    if (tau >= M || j > tau || count[b] <= tau + 1) return;          // uniform over the workgroup
    int f = accepted_idx[b];
    f = f < 0 ? 0 : (f >= K ? K - 1 : f);
    int e = j < tau ? tokens[(static_cast<long long>(b) * K + f) * M + j] : out_tokens[static_cast<long long>(b) * (M + 1) + tau];
    e = e < 0 ? 0 : (e >= V ? V - 1 : e);
    const T *rq = rows_q + ((static_cast<long long>(b) * K + f) * rows_t + j) * static_cast<long long>(V);
    const T *rp = rows_p + ((static_cast<long long>(b) * K + f) * M + j) * static_cast<long long>(V);
    constexpr int PV = Elem<T>::kPerVec;
    RunningSum aq, ap;
    if constexpr (VEC) {
        const int nvec = V / PV;
        for (int v = threadIdx.x; v < nvec; v += kModThreads) {
            float z[PV];
            Elem<T>::unpack(load16_stream(rq + static_cast<long long>(v) * PV), z); aq.add(z, c);
            Elem<T>::unpack(load16_stream(rp + static_cast<long long>(v) * PV), z); ap.add(z, c);
        }
    } else {
        for (int x = threadIdx.x; x < V; x += kModThreads) {
            const float zq[1] = {Elem<T>::scalar(rq + x)}, zp[1] = {Elem<T>::scalar(rp + x)};
            aq.add(zq, c); ap.add(zp, c);
        }
    }
    const float Mq = block_max(aq.m2, sh_f);
    const double Zq = block_sum(static_cast<double>(aq.Z * exp2_fast(aq.m2 - Mq)), sh_d);
    const float Mp = block_max(ap.m2, sh_f);
    const double Zp = block_sum(static_cast<double>(ap.Z * exp2_fast(ap.m2 - Mp)), sh_d);
    if (threadIdx.x == 0) {
        const double l2q = static_cast<double>(Elem<T>::scalar(rq + e)) * static_cast<double>(c) - (static_cast<double>(Mq) + log2(Zq));
        const double l2p = static_cast<double>(Elem<T>::scalar(rp + e)) * static_cast<double>(c) - (static_cast<double>(Mp) + log2(Zp));
        delta[static_cast<long long>(b) * M + j] = (l2q - l2p) * 0.693147180559945309417;
    }
}

// one thread per prefix: sums the log-ratios in position order and shortens the row count
__global__ void k_carry_apply(const int32_t *__restrict__ accepted_len, int M, int batch, const double *__restrict__ delta,
                              double *__restrict__ carry, int32_t *__restrict__ count)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int tau = accepted_len[b], n = count[b];
    if (tau < M && n > tau + 1) {
        double a = carry[b];
        for (int j = 0; j <= tau; ++j) a += delta[static_cast<long long>(b) * M + j];
        carry[b] = a;
        count[b] = n - (tau + 1);
    } else {
        count[b] = 0;                                     // expired: its ratio is not used again
    }
}

template <typename T>
hipError_t launch_carry_typed(const void *rows_q, const void *rows_p, const int32_t *tokens, const int32_t *accepted_len,
                              const int32_t *accepted_idx, const int32_t *out_tokens, int K, int M, int bonus, int V,
                              int batch, float c, double *carry, int32_t *count, double *delta, hipStream_t stream)
{
    const bool vec = (V % Elem<T>::kPerVec) == 0 && reinterpret_cast<uintptr_t>(rows_q) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(rows_p) % 16 == 0;
    const dim3 g(static_cast<unsigned>(M), static_cast<unsigned>(batch));
    if (vec)
        hipLaunchKernelGGL((k_carry_rows<T, true>), g, dim3(kModThreads), 0, stream, static_cast<const T *>(rows_q),
                           static_cast<const T *>(rows_p), tokens, accepted_len, accepted_idx, out_tokens, count, K, M,
                           M + bonus, V, c, delta);
    else
        hipLaunchKernelGGL((k_carry_rows<T, false>), g, dim3(kModThreads), 0, stream, static_cast<const T *>(rows_q),
                           static_cast<const T *>(rows_p), tokens, accepted_len, accepted_idx, out_tokens, count, K, M,
                           M + bonus, V, c, delta);
    hipLaunchKernelGGL(k_carry_apply, dim3((batch + 255) / 256), dim3(256), 0, stream, accepted_len, M, batch, delta, carry,
                       count);
    return hipGetLastError();
}

}  // namespace

size_t modify_workspace_bytes(int batch, int K, int M, int bonus) { return mod_layout(batch, K, M, bonus).total; }

hipError_t launch_modify(const void *target, const void *draft, const int32_t *tokens, int K, int M, int bonus, int V,
                         int batch, int dtype, float c, const double *carry, const int32_t *count, float *out_logq,
                         float *out_logp, double *norm_out, int32_t *fallback_out, char *ws, hipStream_t stream)
{
    return dtype == 1 ? launch_modify_typed<uint16_t>(target, draft, tokens, K, M, bonus, V, batch, c, carry, count,
                                                      out_logq, out_logp, norm_out, fallback_out, ws, stream)
                      : launch_modify_typed<float>(target, draft, tokens, K, M, bonus, V, batch, c, carry, count,
                                                   out_logq, out_logp, norm_out, fallback_out, ws, stream);
}

hipError_t launch_carry_advance(const void *rows_q, const void *rows_p, const int32_t *tokens, const int32_t *accepted_len,
                                const int32_t *accepted_idx, const int32_t *out_tokens, int K, int M, int bonus, int V,
                                int batch, int dtype, float c, double *carry, int32_t *count, double *delta,
                                hipStream_t stream)
{
    return dtype == 1 ? launch_carry_typed<uint16_t>(rows_q, rows_p, tokens, accepted_len, accepted_idx, out_tokens, K, M,
                                                     bonus, V, batch, c, carry, count, delta, stream)
                      : launch_carry_typed<float>(rows_q, rows_p, tokens, accepted_len, accepted_idx, out_tokens, K, M,
                                                  bonus, V, batch, c, carry, count, delta, stream);
}

}  // namespace specgbv
