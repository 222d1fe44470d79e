// Distribution modification (Algorithm 2): the target distribution of the first rows of the
// next iteration.
//
// After an iteration accepted t^tau and drew the final token y, the first count = L - tau - 1
// rows of every new draft use
//     q_new[x] = w[x] / sum_x w[x],   w[x] = q_r[x] max(1 - p_r[x] / (nu q_r[x]), 0)^K
// (Algorithm 2 divided through by the joint probability of the conditioning block: the same
// per-token form as Eq. (pres)), with nu = [q(t^tau, y) / p(t^tau, y)] continued along the new
// draft's own tokens with the original target probabilities.  One workgroup walks the rows of
// one (prefix, draft) pair, because row r needs the normalisers of rows < r; per row it makes
// three passes (statistics, normaliser of w, write), the second and third over lines it has
// just read.  Output: natural-log probabilities in float32 (-inf where the probability is 0).
#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kModThreads = 512;
constexpr int kModWaves = kModThreads / kWave;

struct Pair { double a, b; };

// Two workgroup-wide double sums; every thread gets both (wave-uniform values in SGPR-friendly form).
__device__ __forceinline__ Pair block_sum_pair(double a, double b, double *scratch)
{
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    a = wave_sum(a); b = wave_sum(b);
    __syncthreads();
    if (lane == 0) { scratch[2 * wid] = a; scratch[2 * wid + 1] = b; }
    __syncthreads();
    Pair r{0.0, 0.0};
#pragma unroll
    for (int w = 0; w < kModWaves; ++w) { r.a += scratch[2 * w]; r.b += scratch[2 * w + 1]; }
    return r;
}

// Applies f(x0, zq[8 or fewer], zp[...], n) to consecutive groups of the row pair.
template <typename T, bool VEC, typename F>
__device__ __forceinline__ void for_each_group(const T *rq, const T *rp, int V, F f)
{
    constexpr int PV = Elem<T>::kPerVec;
    if (VEC) {
        const int nvec = V / PV;
        for (int v = threadIdx.x; v < nvec; v += kModThreads) {
            float zq[PV], zp[PV];
            Elem<T>::unpack(load16(rq + static_cast<long long>(v) * PV), zq);
            Elem<T>::unpack(load16(rp + static_cast<long long>(v) * PV), zp);
#pragma unroll
            for (int j = 0; j < PV; ++j) f(v * PV + j, zq[j], zp[j]);
        }
    } else {
        for (int x = threadIdx.x; x < V; x += kModThreads) f(x, Elem<T>::scalar(rq + x), Elem<T>::scalar(rp + x));
    }
}

template <typename T, bool VEC>
__global__ void __launch_bounds__(kModThreads)
k_modify(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens,
         int K, int M, int V, float c, const double *__restrict__ carry_log_nu,
         const int32_t *__restrict__ modify_count, float *__restrict__ out_logq, float *__restrict__ out_logp,
         double *__restrict__ norm_out, int32_t *__restrict__ fallback_out)
{
    __shared__ double sh_d[2 * kModWaves];
    __shared__ float sh_f[2 * kModWaves];
    constexpr double kLn2 = 0.693147180559945309417, kLog2e = 1.44269504088896340736;
    const long long bk = blockIdx.x;
    const int b = static_cast<int>(bk / K);
    int count = modify_count[b];
    count = count < 0 ? 0 : (count > M ? M : count);
    double log2nu = carry_log_nu[b] * kLog2e;

    for (int r = 0; r < M; ++r) {
        const long long row = bk * M + r;
        const T *rq = target + row * static_cast<long long>(V);
        const T *rp = draft + row * static_cast<long long>(V);

        // ---- pass 1: row maxima, then the normalisers relative to them
        float mq = -3.0e38f, mp = -3.0e38f;
        for_each_group<T, VEC>(rq, rp, V, [&](int, float zq, float zp) { mq = fmaxf(mq, zq); mp = fmaxf(mp, zp); });
        mq = wave_max(mq); mp = wave_max(mp);
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0) { sh_f[2 * (threadIdx.x / kWave)] = mq; sh_f[2 * (threadIdx.x / kWave) + 1] = mp; }
        __syncthreads();
        mq = sh_f[0]; mp = sh_f[1];
#pragma unroll
        for (int w = 1; w < kModWaves; ++w) { mq = fmaxf(mq, sh_f[2 * w]); mp = fmaxf(mp, sh_f[2 * w + 1]); }
        const float ref_q = mq * c, ref_p = mp * c;
        float Zq = 0.0f, Zp = 0.0f;
        for_each_group<T, VEC>(rq, rp, V, [&](int, float zq, float zp) {
            Zq += exp2_fast(fmaf(zq, c, -ref_q));
            Zp += exp2_fast(fmaf(zp, c, -ref_p));
        });
        const Pair Z = block_sum_pair(static_cast<double>(Zq), static_cast<double>(Zp), sh_d);
        const double lse2_q = static_cast<double>(ref_q) + log2(Z.a), lse2_p = static_cast<double>(ref_p) + log2(Z.b);
        // log2 q[x] = fma(z, c, -sq) - dq with a float reference sq and its float64 remainder dq
        const float sq = static_cast<float>(lse2_q), sp = static_cast<float>(lse2_p);
        const float dq = static_cast<float>(lse2_q - static_cast<double>(sq));
        const float dp = static_cast<float>(lse2_p - static_cast<double>(sp));

        float *oq = out_logq + row * static_cast<long long>(V);
        float *op = out_logp ? out_logp + row * static_cast<long long>(V) : nullptr;
        const bool modified = r < count;
        double W = 1.0;
        int fb = 0;
        if (modified) {
            // ---- pass 2: normaliser of the weights
            const RatioConst rc(lse2_p - lse2_q + log2nu);
            float acc = 0.0f;
            for_each_group<T, VEC>(rq, rp, V, [&](int, float zq, float zp) {
                const float eq = exp2_fast(fmaf(zq, c, -sq));
                acc = fmaf(eq, powi_uniform(rc.one_minus_ratio(zp - zq, c), K), acc);
            });
            const Pair S = block_sum_pair(static_cast<double>(acc), 0.0, sh_d);
            W = S.a * exp2(static_cast<double>(sq) - lse2_q);
            fb = !(W > 0.0);
            if (fb) W = 1.0;
            // ---- pass 3: ln q_new = ln q + K ln t - ln W (all-zero weights: the row stays q)
            const float log2W = fb ? 0.0f : static_cast<float>(log2(S.a));     // relative to 2^sq like acc
            const float Kf = static_cast<float>(K);
            for_each_group<T, VEC>(rq, rp, V, [&](int x, float zq, float zp) {
                const float x2 = fmaf(zq, c, -sq);
                float l2;
                if (fb) l2 = x2 - dq;
                else l2 = fmaf(Kf, __log2f(rc.one_minus_ratio(zp - zq, c)), x2) - log2W;
                oq[x] = l2 * static_cast<float>(kLn2);
                if (op) op[x] = (fmaf(zp, c, -sp) - dp) * static_cast<float>(kLn2);
            });
        } else {
            for_each_group<T, VEC>(rq, rp, V, [&](int x, float zq, float zp) {
                oq[x] = (fmaf(zq, c, -sq) - dq) * static_cast<float>(kLn2);
                if (op) op[x] = (fmaf(zp, c, -sp) - dp) * static_cast<float>(kLn2);
            });
        }
        if (threadIdx.x == 0) {
            if (norm_out) norm_out[row] = W;
            if (fallback_out) fallback_out[row] = fb;
        }
        // extend the block by this row's token
        int tok = tokens[row];
        tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
        const double tq = static_cast<double>(Elem<T>::scalar(rq + tok)) * static_cast<double>(c) - lse2_q;
        const double tp = static_cast<double>(Elem<T>::scalar(rp + tok)) * static_cast<double>(c) - lse2_p;
        log2nu += tq - tp;
    }
}

template <typename T>
hipError_t launch_modify_typed(const void *target, const void *draft, const int32_t *tokens, int K, int M, int V,
                               int batch, float c, const double *carry, const int32_t *count, float *out_logq,
                               float *out_logp, double *norm_out, int32_t *fallback_out, hipStream_t stream)
{
    const bool vec = (V % Elem<T>::kPerVec) == 0 && reinterpret_cast<uintptr_t>(target) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(draft) % 16 == 0;
    const dim3 grid(static_cast<unsigned>(static_cast<long long>(batch) * K));
    if (vec)
        hipLaunchKernelGGL((k_modify<T, true>), grid, dim3(kModThreads), 0, stream, static_cast<const T *>(target),
                           static_cast<const T *>(draft), tokens, K, M, V, c, carry, count, out_logq, out_logp,
                           norm_out, fallback_out);
    else
        hipLaunchKernelGGL((k_modify<T, false>), grid, dim3(kModThreads), 0, stream, static_cast<const T *>(target),
                           static_cast<const T *>(draft), tokens, K, M, V, c, carry, count, out_logq, out_logp,
                           norm_out, fallback_out);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_modify(const void *target, const void *draft, const int32_t *tokens, int K, int M, int V, int batch,
                         int dtype, float c, const double *carry, const int32_t *count, float *out_logq,
                         float *out_logp, double *norm_out, int32_t *fallback_out, hipStream_t stream)
{
    return dtype == 1 ? launch_modify_typed<uint16_t>(target, draft, tokens, K, M, V, batch, c, carry, count, out_logq,
                                                      out_logp, norm_out, fallback_out, stream)
                      : launch_modify_typed<float>(target, draft, tokens, K, M, V, batch, c, carry, count, out_logq,
                                                   out_logp, norm_out, fallback_out, stream);
}

}  // namespace specgbv
