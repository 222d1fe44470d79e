// Schedule "chain": every (target, draft) row pair is read from HBM once.
//
// One 512-thread workgroup owns one (prefix, draft) pair and walks its L row pairs in
// order.  A row pair stays on chip between the two sweeps that need it:
//
//   sweep 1  soft-max statistics  Z_q = sum_x 2^(c z_q[x] - ref_q),  Z_p likewise
//   sweep 2  the vocabulary sum of Eq. (hik) divided by q(x^i),
//              s_i = sum_x q_i[x] max(1 - p_i[x] / (nu_i q_i[x]), 0)^K,
//            which needs the row's own normalisers and nu_i from the rows before it
//
// Each thread keeps its 16-byte vectors of the row pair in RS VGPR slots (all of them
// full: the host picks RS <= V-in-vectors / 512) and up to kLdsSlots LDS slots; with
// RS = 23 that is 32 slots of a (q, p) vector pair = 1 KiB per thread, 512 KiB per
// workgroup: one bf16 row pair of 128K entries.  Vectors beyond that are read a second
// time in sweep 2 (they were just streamed, so they mostly come from cache).  While
// sweep 2 consumes a register slot, the load of the next row's vector for that slot is
// issued into the same registers, so HBM latency is hidden behind arithmetic.  Because
// the chain is walked inside one workgroup, nu_i is available without any exchange
// between workgroups.
//
// The reference exponents ref_q, ref_p are the workgroup-wide maxima over each thread's
// first vector (a 4096-entry sample) instead of the exact row maxima; should a row
// overflow float32 with that reference (possible only for extremely peaked rows), its
// statistics are recomputed from memory with the exact maximum.
#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kChainThreads = 512;
constexpr int kChainWaves = kChainThreads / kWave;
constexpr int kLdsSlots = 9;

// t[j] <- t[j]^K.  KP > 0 fixes K at compile time; KP = 0 takes the wave-uniform K >= 1.
template <int KP, int N>
__device__ __forceinline__ void pow_inplace(float (&t)[N], int K)
{
    if (KP == 1) return;
    if (KP == 2 || KP == 4 || KP == 8 || KP == 16) {
#pragma unroll
        for (int j = 0; j < N; ++j) {
            float a = t[j] * t[j];
            if (KP >= 4) a = a * a;
            if (KP >= 8) a = a * a;
            if (KP >= 16) a = a * a;
            t[j] = a;
        }
        return;
    }
    if (KP == 3) {
#pragma unroll
        for (int j = 0; j < N; ++j) t[j] = t[j] * t[j] * t[j];
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

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_cvoid;

struct RowConsts {
    float c;
    float nref_q, nref_p;    // minus the reference exponents
    float C2_hi, neg_kappa;  // ratio constants (see RatioConst)
    int K;
};

template <typename T>
__device__ __forceinline__ void sweep1_vec(const U4 &q, const U4 &p, const RowConsts &rc, float &Zq, float &Zp)
{
    constexpr int PV = Elem<T>::kPerVec;
    float zq[PV], zp[PV];
    Elem<T>::unpack(q, zq);
    Elem<T>::unpack(p, zp);
    float a = 0.0f, b = 0.0f;
#pragma unroll
    for (int j = 0; j < PV; ++j) {
        a += exp2_fast(fmaf(zq[j], rc.c, rc.nref_q));
        b += exp2_fast(fmaf(zp[j], rc.c, rc.nref_p));
    }
    Zq += a; Zp += b;
}

template <typename T, int KP>
__device__ __forceinline__ void sweep2_vec(const U4 &q, const U4 &p, const RowConsts &rc, float &acc)
{
    constexpr int PV = Elem<T>::kPerVec;
    float zq[PV], zp[PV], t[PV];
    // Opaque copies: without them the compiler keeps the floats that sweep 1 unpacked from
    // these registers alive until here, which doubles the footprint of bf16 rows.
    U4 qq = q, pp = p;
    asm volatile("" : "+v"(qq.x), "+v"(qq.y), "+v"(qq.z), "+v"(qq.w));
    asm volatile("" : "+v"(pp.x), "+v"(pp.y), "+v"(pp.z), "+v"(pp.w));
    Elem<T>::unpack(qq, zq);
    Elem<T>::unpack(pp, zp);
#pragma unroll
    for (int j = 0; j < PV; ++j) {
        const float r = exp2_fast(fmaf(zp[j] - zq[j], rc.c, -rc.C2_hi));
        t[j] = __builtin_amdgcn_fmed3f(fmaf(r, rc.neg_kappa, 1.0f), 0.0f, 1.0f);
    }
    pow_inplace<KP>(t, rc.K);
    float a = 0.0f;
#pragma unroll
    for (int j = 0; j < PV; ++j) a = fmaf(exp2_fast(fmaf(zq[j], rc.c, rc.nref_q)), t[j], a);
    acc += a;
}

// 16-byte vector number slot*512 + lane of a row: wave-uniform base plus a 32-bit lane offset.
template <typename T>
__device__ __forceinline__ U4 load_slot(const T *row, int slot, unsigned lane)
{
    const U4 *base = reinterpret_cast<const U4 *>(row) + static_cast<size_t>(slot) * kChainThreads;
    return base[lane];
}

template <typename T>
__device__ __forceinline__ float vec_max(const U4 &v)
{
    constexpr int PV = Elem<T>::kPerVec;
    float z[PV];
    Elem<T>::unpack(v, z);
    float m = z[0];
#pragma unroll
    for (int j = 1; j < PV; ++j) m = fmaxf(m, z[j]);
    return m;
}

// Two workgroup-wide double sums with one pair of barriers.
__device__ __forceinline__ void block_sum2(double &a, double &b, double *scratch)
{
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    a = wave_sum(a); b = wave_sum(b);
    __syncthreads();
    if (lane == 0) { scratch[2 * wid] = a; scratch[2 * wid + 1] = b; }
    __syncthreads();
    double ra = 0.0, rb = 0.0;
#pragma unroll
    for (int w = 0; w < kChainWaves; ++w) { ra += scratch[2 * w]; rb += scratch[2 * w + 1]; }
    a = ra; b = rb;
}

__device__ __forceinline__ void block_max2(float &a, float &b, float *scratch)
{
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    a = wave_max(a); b = wave_max(b);
    __syncthreads();
    if (lane == 0) { scratch[2 * wid] = a; scratch[2 * wid + 1] = b; }
    __syncthreads();
    float ra = scratch[0], rb = scratch[1];
#pragma unroll
    for (int w = 1; w < kChainWaves; ++w) { ra = fmaxf(ra, scratch[2 * w]); rb = fmaxf(rb, scratch[2 * w + 1]); }
    a = ra; b = rb;
}

// log2 of a positive finite double from its exponent and a float log of the mantissa
// (absolute error about 1e-7).
__device__ __forceinline__ double log2_cheap(double z)
{
    int e;
    const double m = frexp(z, &e);              // z = m * 2^e, m in [0.5, 1)
    return static_cast<double>(e) + static_cast<double>(__log2f(static_cast<float>(m)));
}

// Exact-maximum statistics of one row straight from memory (overflow fallback).
template <typename T>
__device__ __noinline__ void exact_row_stats(const T *row, int nvec, float c, float &ref_out, double &Z_out,
                                             float *sh_f, double *sh_d)
{
    constexpr int PV = Elem<T>::kPerVec;
    float m = -3.0e38f;
    for (int v = threadIdx.x; v < nvec; v += kChainThreads)
        m = fmaxf(m, vec_max<T>(load16(row + static_cast<long long>(v) * PV)));
    float dummy = m;
    block_max2(m, dummy, sh_f);
    const float ref = m * c;
    float Z = 0.0f;
    for (int v = threadIdx.x; v < nvec; v += kChainThreads) {
        float z[PV];
        Elem<T>::unpack(load16(row + static_cast<long long>(v) * PV), z);
#pragma unroll
        for (int j = 0; j < PV; ++j) Z += exp2_fast(fmaf(z[j], c, -ref));
    }
    double a = static_cast<double>(Z), b = 0.0;
    block_sum2(a, b, sh_d);
    ref_out = ref; Z_out = a;
}

template <typename T, int KP, int RS>
__global__ void __launch_bounds__(kChainThreads)
k_chain(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens,
        int K, int L, int V, float c, RowStat *__restrict__ stats, double *__restrict__ s_out, int dbg)
{
    __shared__ U4 lds_q[kLdsSlots][kChainThreads];
    __shared__ U4 lds_p[kLdsSlots][kChainThreads];
    __shared__ double sh_d[2 * kChainWaves];
    __shared__ float sh_f[2 * kChainWaves];

    constexpr int PV = Elem<T>::kPerVec;
    const unsigned tid = threadIdx.x;
    const long long bk = blockIdx.x;                       // b*K + k
    const int nvec = V / PV;                               // host guarantees nvec >= RS * 512
    const int rem = nvec - static_cast<int>(tid);          // slot j holds a vector of this thread iff j*512 < rem
    const int nslots = (dbg & 2) ? RS : (nvec + kChainThreads - 1) / kChainThreads;
    const T *trow0 = target + bk * (L + 1) * static_cast<long long>(V);
    const T *drow0 = draft + bk * L * static_cast<long long>(V);

    if (dbg & 4) {                                         // experiment: de-phase neighbouring workgroups
        const int naps = (blockIdx.x & 3) * ((dbg >> 4) & 15);
        for (int i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(127);
    }
    U4 rq[RS], rp[RS];
#pragma unroll
    for (int j = 0; j < RS; ++j) {
        rq[j] = load_slot(trow0, j, tid);
        rp[j] = load_slot(drow0, j, tid);
    }

    double log2nu = 0.0;                                   // block ratio of the rows before row r
    for (int r = 0; r < L; ++r) {
        const T *qrow = trow0 + static_cast<long long>(r) * V;
        const T *prow = drow0 + static_cast<long long>(r) * V;

        // reference exponents from the first vector of every thread
        float mq = vec_max<T>(rq[0]), mp = vec_max<T>(rp[0]);
        block_max2(mq, mp, sh_f);
        RowConsts rc;
        rc.c = c; rc.K = K;
        rc.nref_q = -(mq * c); rc.nref_p = -(mp * c);

        // ---- sweep 1
        // The LDS slots of this row are filled by asynchronous global->LDS loads (no VGPRs,
        // one 16-byte element per lane, written to consecutive LDS addresses of the wave)
        // while the register slots are being processed.
        const int lds_end = nslots < RS + kLdsSlots ? nslots : RS + kLdsSlots;
        if (!(dbg & 32)) {
            for (int j = RS; j < lds_end; ++j) {
                if (j * kChainThreads < rem) {
                    const unsigned wbase = tid & ~(kWave - 1u);
                    __builtin_amdgcn_global_load_lds(
                        (glb_cvoid *)(reinterpret_cast<const U4 *>(qrow) + static_cast<size_t>(j) * kChainThreads + tid),
                        (lds_void *)&lds_q[j - RS][wbase], 16, 0, 0);
                    __builtin_amdgcn_global_load_lds(
                        (glb_cvoid *)(reinterpret_cast<const U4 *>(prow) + static_cast<size_t>(j) * kChainThreads + tid),
                        (lds_void *)&lds_p[j - RS][wbase], 16, 0, 0);
                }
            }
        }
        float Zq = 0.0f, Zp = 0.0f;
#pragma unroll
        for (int j = 0; j < RS; ++j) {
            if (dbg & 8) { Zq += __uint_as_float((rq[j].x ^ rq[j].y ^ rq[j].z ^ rq[j].w) & 0x3fffffffu); Zp += __uint_as_float((rp[j].x ^ rp[j].w) & 0x3fffffffu); }
            else sweep1_vec<T>(rq[j], rp[j], rc, Zq, Zp);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the LDS fills have landed
        for (int j = RS; j < nslots; ++j) {
            if (j * kChainThreads < rem) {
                U4 q, p;
                if (j < lds_end && !(dbg & 32)) { q = lds_q[j - RS][tid]; p = lds_p[j - RS][tid]; }
                else {
                    q = load_slot(qrow, j, tid); p = load_slot(prow, j, tid);
                    if (j < lds_end) { lds_q[j - RS][tid] = q; lds_p[j - RS][tid] = p; }
                }
                sweep1_vec<T>(q, p, rc, Zq, Zp);
            }
        }
        double Zq_tot = static_cast<double>(Zq), Zp_tot = static_cast<double>(Zp);
        block_sum2(Zq_tot, Zp_tot, sh_d);
        float ref_q = -rc.nref_q, ref_p = -rc.nref_p;
        if (!(Zq_tot < 1.0e37) || !(Zq_tot > 0.0)) {       // float32 overflow with the sample reference
            exact_row_stats<T>(qrow, nvec, c, ref_q, Zq_tot, sh_f, sh_d);
            rc.nref_q = -ref_q;                            // sweep 2 reuses the target reference
        }
        if (!(Zp_tot < 1.0e37) || !(Zp_tot > 0.0)) exact_row_stats<T>(prow, nvec, c, ref_p, Zp_tot, sh_f, sh_d);

        const double lse2_q = static_cast<double>(ref_q) + log2_cheap(Zq_tot);
        const double lse2_p = static_cast<double>(ref_p) + log2_cheap(Zp_tot);
        int tok = tokens[bk * L + r];
        tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
        const double tok2_q = static_cast<double>(Elem<T>::scalar(qrow + tok)) * static_cast<double>(c);
        const double tok2_p = static_cast<double>(Elem<T>::scalar(prow + tok)) * static_cast<double>(c);
        if (tid == 0) {
            RowStat st;
            st.lse2_q = lse2_q; st.lse2_p = lse2_p; st.tok2_q = tok2_q; st.tok2_p = tok2_p;
            stats[bk * L + r] = st;
        }

        // ---- sweep 2 (rows 1..L-1; row 0 carries no Eq. (hik) sum) and loads of the next row.
        // After the last row the "next row" loads all read one 16-byte line of the current
        // row (lane offset 0) so that the register slots are written on every path.
        const bool more = r + 1 < L && !(dbg & 1);
        const bool sum_row = r >= 1;
        const T *qnext = more ? qrow + V : qrow, *pnext = more ? prow + V : prow;
        const unsigned lane_next = more ? tid : 0u;
        const double C2 = lse2_p - lse2_q + log2nu;
        rc.C2_hi = static_cast<float>(C2);
        const double dk = (static_cast<double>(rc.C2_hi) - C2) * 0.693147180559945309417;
        rc.neg_kappa = (dk > -0.25 && dk < 0.25) ? -static_cast<float>(1.0 + dk + 0.5 * dk * dk) : -1.0f;
        float acc = 0.0f;
#pragma unroll
        for (int j = 0; j < RS; ++j) {
            if (dbg & 8) acc += __uint_as_float((rq[j].y ^ rp[j].z) & 0x3fffffffu);
            else if (sum_row) sweep2_vec<T, KP>(rq[j], rp[j], rc, acc);
            unsigned lane = lane_next;
            asm volatile("" : "+v"(lane) : "v"(acc));       // keep the loads behind this slot's arithmetic
            rq[j] = load_slot(qnext, j, lane);
            rp[j] = load_slot(pnext, j, lane);
        }
        if (sum_row) {
            for (int j = RS; j < nslots; ++j) {
                if (j * kChainThreads < rem) {
                    U4 q, p;
                    if (j < RS + kLdsSlots) { q = lds_q[j - RS][tid]; p = lds_p[j - RS][tid]; }
                    else { q = load_slot(qrow, j, tid); p = load_slot(prow, j, tid); }
                    sweep2_vec<T, KP>(q, p, rc, acc);
                }
            }
            double s_tot = static_cast<double>(acc), unused = 0.0;
            block_sum2(s_tot, unused, sh_d);
            if (tid == 0) s_out[bk * L + r] = s_tot / Zq_tot;
        }
        log2nu += (tok2_q - lse2_q) - (tok2_p - lse2_p);
    }
}

template <typename T, int KP>
hipError_t launch_kp(const Problem &p)
{
    RowStat *stats = reinterpret_cast<RowStat *>(p.ws + p.lay.stats);
    double *s = reinterpret_cast<double *>(p.ws + p.lay.s);
    const dim3 grid(static_cast<unsigned>(static_cast<long long>(p.batch) * p.K));
    const T *target = static_cast<const T *>(p.target);
    const T *draft = static_cast<const T *>(p.draft);
    const int full_slots = (p.V / Elem<T>::kPerVec) / kChainThreads;
#define SPECGBV_LAUNCH(RS)                                                                              \
    hipLaunchKernelGGL((k_chain<T, KP, RS>), grid, dim3(kChainThreads), 0, p.stream, target, draft,    \
                       p.tokens, p.K, p.L, p.V, p.c, stats, s, p.debug)
    if (full_slots >= 23) SPECGBV_LAUNCH(23);
    else if (full_slots >= 15) SPECGBV_LAUNCH(15);
    else SPECGBV_LAUNCH(7);
#undef SPECGBV_LAUNCH
    return hipGetLastError();
}

template <typename T>
hipError_t launch_typed(const Problem &p)
{
    switch (p.K) {
    case 8: return launch_kp<T, 8>(p);
    default: return launch_kp<T, 0>(p);
    }
}

}  // namespace

bool chain_supported(const Problem &p)
{
    const int pv = p.dtype == 1 ? 8 : 4;
    return p.V % pv == 0 && (p.V / pv) >= 7 * kChainThreads &&
           reinterpret_cast<uintptr_t>(p.target) % 16 == 0 && reinterpret_cast<uintptr_t>(p.draft) % 16 == 0;
}

hipError_t launch_chain_main(const Problem &p)
{
    return p.dtype == 1 ? launch_typed<uint16_t>(p) : launch_typed<float>(p);
}

}  // namespace specgbv
