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
// The reference exponents ref_q, ref_p are the scaled logits of the row's drafted token
// instead of the exact row maxima; should a row's sum exceed 2^30 times the token's weight
// (a drafted token of probability below 1e-9: very low temperatures, extremely peaked rows;
// float32 overflow is the extreme case), its statistics are recomputed from memory with the
// exact maximum, because exponents that large lose absolute accuracy in float32.
//
// Pending distribution modifications (Algorithm 2 applied on the fly, PEND variants): once a
// row's statistics are known and while the whole row pair is still on chip, every level that
// modifies the row gets its normaliser from one more sweep over the on-chip copy (no memory
// traffic), and so does the row's Eq. (hik) sum against the modified row; such a row's slots
// are then simply reloaded in the next iteration.  Needs the whole row pair on chip.
#include <utility>

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

// Asynchronous 16-byte-per-lane load from global memory straight into LDS: lane l of the
// wave writes LDS bytes [dst + 16 l, dst + 16 l + 16), dst wave-uniform.  Completion is
// tracked by vmcnt only.  Issued as inline assembly: the compiler otherwise treats the
// instruction as a flat access that may touch LDS and from then on turns every vector-memory
// wait into vmcnt(0), which would drain the load pipeline at each use of a loaded register.
// (Its own vmcnt arithmetic does not see these loads, so its waits are conservative.)
__device__ __forceinline__ void lds_fill16(const void *src_base_uniform, unsigned lane_byte_off, unsigned lds_dst_wave_uniform)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(lane_byte_off), "s"(src_base_uniform), "s"(lds_dst_wave_uniform)
                 : "memory", "m0");
}

struct RowConsts {
    float c;
    float nref_q, nref_p;    // minus the reference exponents
    float C2_hi, neg_kappa;  // ratio constants (see RatioConst)
    int K;
};

// `tok_slot` (uniform): this slot of the row holds the drafted token's vector, in the lane for which `tok_mine`
// holds.  That vector's weights are summed apart, from a copy fetched with the token's logits (see the row loop):
// next to the token's weight, which is one, the float32 sums of its thread would lose the other entries' low bits,
// and a row whose drafted token has probability 0.9999 needs exactly those (its remaining mass is what 1 - P and
// 1 - Q in Eq. (hik) are made of).
template <typename T>
__device__ __forceinline__ void sweep1_vec(const U4 &q, const U4 &p, const RowConsts &rc, float &Zq, float &Zp,
                                           bool tok_slot = false, bool tok_mine = false)
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
    if (!(tok_slot && tok_mine)) {
        asm volatile("");                       // (keeps this a masked block: two adds, and scalar work for the mask)
        Zq += a; Zp += b;
    }
}

template <typename T, int KP>
__device__ __forceinline__ void sweep2_vec(const U4 &q, const U4 &p, const RowConsts &rc, float &acc)
{
    constexpr int PV = Elem<T>::kPerVec;
    float zq[PV], zp[PV], t[PV];
    Elem<T>::unpack(q, zq);
    Elem<T>::unpack(p, zp);
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

// 16-byte vector at a wave-uniform base plus a 32-bit per-lane byte offset (scalar-base addressing:
// no per-load vector address arithmetic, no 64-bit address registers).
__device__ __forceinline__ U4 load_vec(const void *base_uniform, unsigned lane_byte_off)
{
    // The base is pinned to a scalar register pair: otherwise the compiler folds it into a
    // 64-bit per-lane address first and then spends vector adds on each slot's constant.
    // (The pointer keeps its global address space through the opaque copy; a generic pointer
    // would turn the access into a flat load.)
    typedef unsigned int V4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(1))) char *GlobalBytes;
    GlobalBytes b = (GlobalBytes)base_uniform;
    asm volatile("" : "+s"(b));
    const V4 v = __builtin_nontemporal_load((const __attribute__((address_space(1))) V4 *)(b + lane_byte_off));
    return U4{v.x, v.y, v.z, v.w};
}
template <typename T>
__device__ __forceinline__ U4 load_slot(const T *row, int slot, unsigned lane)
{
    return load_vec(reinterpret_cast<const char *>(row) + static_cast<size_t>(slot) * (kChainThreads * 16), lane * 16u);
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

// Three workgroup-wide double sums with one pair of barriers.
__device__ __forceinline__ void block_sum3(double &a, double &b, double &d, double *scratch)
{
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    a = wave_sum(a); b = wave_sum(b); d = wave_sum(d);
    __syncthreads();
    if (lane == 0) { scratch[3 * wid] = a; scratch[3 * wid + 1] = b; scratch[3 * wid + 2] = d; }
    __syncthreads();
    double ra = 0.0, rb = 0.0, rd = 0.0;
#pragma unroll
    for (int w = 0; w < kChainWaves; ++w) { ra += scratch[3 * w]; rb += scratch[3 * w + 1]; rd += scratch[3 * w + 2]; }
    a = ra; b = rb; d = rd;
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

// A workgroup-uniform double moved to scalar registers, so that values carried across the row
// loop do not occupy (or spill) vector registers.
__device__ __forceinline__ double uniform_d(double v)
{
    const long long b = __double_as_longlong(v);
    const unsigned lo = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(b));
    const unsigned hi = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(static_cast<unsigned long long>(b) >> 32));
    return __longlong_as_double(static_cast<long long>((static_cast<unsigned long long>(hi) << 32) | lo));
}

// Exact-maximum statistics of one row straight from memory (overflow fallback).  Results are
// returned by value: reference parameters of a function that is not inlined would pin the
// caller's variables to scratch memory for the whole kernel.
struct ExactStats { float ref; double Z; };
template <typename T>
__device__ __noinline__ ExactStats exact_row_stats(const T *row, int nvec, float c, double *sh_d)
{
    float *sh_f = reinterpret_cast<float *>(sh_d);
    constexpr int PV = Elem<T>::kPerVec;
    float m = -3.0e38f;
    for (int v = threadIdx.x; v < nvec; v += kChainThreads)
        m = fmaxf(m, vec_max<T>(load16_stream(row + static_cast<long long>(v) * PV)));
    float dummy = m;
    block_max2(m, dummy, sh_f);
    const float ref = m * c;
    float Z = 0.0f;
    for (int v = threadIdx.x; v < nvec; v += kChainThreads) {
        float z[PV];
        Elem<T>::unpack(load16_stream(row + static_cast<long long>(v) * PV), z);
#pragma unroll
        for (int j = 0; j < PV; ++j) Z += exp2_fast(fmaf(z[j], c, -ref));
    }
    double a = static_cast<double>(Z), b = 0.0;
    block_sum2(a, b, sh_d);
    return ExactStats{ref, a};
}

constexpr int kExcessThreads = 256;

// excess_needed as a function of its own: called by one thread for the few rows that pass excess_wanted, its float64
// registers would otherwise be taken from the ones that hold the row pair.
__device__ __noinline__ bool excess_needed_call(double log2nu, double log2P, double s, int K)
{
    return excess_needed(log2nu, log2P, s, K);
}

// s with the drafted token's term exchanged for its float64 value (see token_term), likewise a function of its own:
// s_tot the row's float32-summed terms and in_sweep the token's among them, both relative to the reference that the
// normaliser 1 / inv_Zq is relative to.
__device__ __noinline__ double token_term_call(double s_tot, float in_sweep, double inv_Zq, const TokenTerm *tt, int K)
{
    return (s_tot - static_cast<double>(in_sweep)) * inv_Zq + token_term(tt->log2q, tt->log2r, K);
}

// Rows a workgroup of k_chain hands to k_chain_excess: entry 0 of its list is their number, then their row indices.
// A list has room for every row the workgroup sums.
inline int later_list_entries(long long nchains, long long grid, int L)
{
    return 1 + static_cast<int>((nchains + grid - 1) / grid) * (L > 1 ? L - 1 : 0);
}

constexpr int kLag = 6;    // slots between the load of a vector and its first use
constexpr double kTokenRefLimit = 1073741824.0;   // 2^30: largest row sum accepted relative to the drafted token's weight

struct LdsSlots {
    U4 *all;                 // [kLdsSlots][2][kChainThreads]: slot s, half 0 = target vectors, half 1 = draft vectors
    unsigned wave_base;      // LDS byte address of this wave's 1 KiB window in slot 0, half 0
};
__device__ __forceinline__ const U4 &lds_vec(const LdsSlots &lds, int s, int half, unsigned t)
{
    return lds.all[(s * 2 + half) * kChainThreads + t];
}

template <typename T>
struct StepCtx {
    const T *qnew, *pnew;
    const RowConsts &rc_sum, &rc_new;
    unsigned tid, off_new;   // thread index; byte offset of this lane's vector within a slot of the new row (0 after the last row)
    int nvec, rem, n_on;
    bool do_new, do_sum;
    int tok_slot;            // slot of the new row that holds the drafted token's vector (uniform)
    bool tok_mine;           // ... and whether this lane's vector of that slot is the one
};

// Order in which the on-chip slots of a row are visited: the LDS slots first, from the highest down (slots a short
// row leaves unused thus come first and the used ones sit right in front of the register slots), then the register
// slots.  The compiler counts the loads it issued itself when it places the wait for a register slot; it cannot see
// the asynchronous global->LDS fills, which are inline assembly.  With the fills at the start of the row no fill
// follows a register load inside an iteration, so the compiler's count for every register slot is exact, and it
// never waits for more than the slot it is about to read.
template <int RS>
constexpr int slot_at(int i) { return i < kLdsSlots ? RS + kLdsSlots - 1 - i : i - kLdsSlots; }

// Step I of the slot pipeline (all indices are compile-time constants so that the slot arrays stay in registers):
// sweep 2 of the old row on slot J = slot_at(I), the load of the new row into slot J, and sweep 1 of the new row
// on the slot of step I - kLag.  Register slots are waited for by the compiler.  LDS slots were filled by
// asynchronous global->LDS loads, so a manual wait precedes their first read: every one of the kLag steps after the
// fill of a used LDS slot issues two vector-memory operations (the used LDS slots are contiguous and the register
// slots follow them), none of which may be pending once the fill has landed.
template <typename T, int KP, int RS, int I>
__device__ __forceinline__ void pipeline_step(const StepCtx<T> &cx, U4 (&rq)[RS], U4 (&rp)[RS],
                                              const LdsSlots &lds, float &Zq, float &Zp, float &acc)
{
    constexpr int NS = RS + kLdsSlots;
    static_assert(RS >= kLag, "the steps after the last LDS fill must all be register loads");
    constexpr size_t kSlotBytes = static_cast<size_t>(kChainThreads) * 16;
    // Opaque copies: everything derived from them is recomputed per step instead of being
    // hoisted out of the row loop and kept (or spilled) across it.
    unsigned t = cx.tid, off = cx.off_new;
    asm volatile("" : "+v"(t), "+v"(off));
    if constexpr (I < NS) {
        constexpr int J = slot_at<RS>(I);
        if constexpr (J < RS) {
            // Opaque touch of the slot: without it the compiler keeps the floats that sweep 1
            // unpacked from these registers alive until sweep 2, which doubles the footprint of
            // bf16 rows.
            asm volatile("" : "+v"(rq[J].x), "+v"(rq[J].y), "+v"(rq[J].z), "+v"(rq[J].w));
            asm volatile("" : "+v"(rp[J].x), "+v"(rp[J].y), "+v"(rp[J].z), "+v"(rp[J].w));
            if (cx.do_sum) sweep2_vec<T, KP>(rq[J], rp[J], cx.rc_sum, acc);
            asm volatile("" : "+v"(off) : "v"(acc));        // keep the loads behind this slot's arithmetic
            rq[J] = load_vec(reinterpret_cast<const char *>(cx.qnew) + J * kSlotBytes, off);
            rp[J] = load_vec(reinterpret_cast<const char *>(cx.pnew) + J * kSlotBytes, off);
        } else if (J < cx.n_on) {
            if (cx.do_sum && J * kChainThreads < cx.rem)
                sweep2_vec<T, KP>(lds_vec(lds, J - RS, 0, t), lds_vec(lds, J - RS, 1, t), cx.rc_sum, acc);
            if (cx.do_new) {
                // every lane loads (lanes past the row end re-read its last vector) so that
                // all waves issue the same number of vector-memory operations
                const unsigned last = static_cast<unsigned>(cx.nvec - 1 - J * kChainThreads) * 16u;   // uniform
                unsigned o = off < last ? off : last;
                asm volatile("" : "+v"(o) : "v"(acc));
                lds_fill16(reinterpret_cast<const char *>(cx.qnew) + J * kSlotBytes, o,
                           lds.wave_base + (J - RS) * 2 * kChainThreads * 16);
                lds_fill16(reinterpret_cast<const char *>(cx.pnew) + J * kSlotBytes, o,
                           lds.wave_base + ((J - RS) * 2 + 1) * kChainThreads * 16);
            }
        }
    }
    constexpr int II = I - kLag;                            // lagged sweep 1 of the new row
    if constexpr (II >= 0 && II < NS) {
        constexpr int JJ = slot_at<RS>(II);
        if constexpr (JJ < RS) {
            if (cx.do_new) sweep1_vec<T>(rq[JJ], rp[JJ], cx.rc_new, Zq, Zp, JJ == cx.tok_slot, cx.tok_mine);
        } else {
            // (the loads of this step are issued before the wait that counts them)
            __builtin_amdgcn_sched_barrier(0);
            if (cx.do_new && JJ < cx.n_on) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kLag) : "memory");
                if (JJ * kChainThreads < cx.rem)
                    sweep1_vec<T>(lds_vec(lds, JJ - RS, 0, t), lds_vec(lds, JJ - RS, 1, t), cx.rc_new, Zq, Zp,
                                  JJ == cx.tok_slot, cx.tok_mine);
            }
        }
    }
}

template <typename T, int KP, int RS, int... Js>
__device__ __forceinline__ void run_steps(std::integer_sequence<int, Js...>, const StepCtx<T> &cx, U4 (&rq)[RS],
                                          U4 (&rp)[RS], const LdsSlots &lds, float &Zq, float &Zp, float &acc)
{
    (pipeline_step<T, KP, RS, Js>(cx, rq, rp, lds, Zq, Zp, acc), ...);
}

// log2 of a positive finite double from its exponent and a float log of the mantissa
// (absolute error about 1e-7).
__device__ __forceinline__ double log2_cheap(double z)
{
    int e;
    const double m = frexp(z, &e);              // z = m * 2^e, m in [0.5, 1)
    return static_cast<double>(e) + static_cast<double>(__log2f(static_cast<float>(m)));
}

// log2 of a positive finite double to float64 accuracy: the float logarithm above, then one Newton step on
// 2^y = m with the small float64 exponential (the error is squared: about 1e-14).  A function of its own, so that
// its float64 constants stay out of the kernel's loop, whose registers hold a whole row pair.  A row's
// log-normaliser enters every block ratio after it, and sub-block acceptance probabilities can be several times
// more sensitive to the block ratio than 1:1, so the 1e-7 of the float logarithm is not good enough there.
__device__ __noinline__ double log2_refined(double z)
{
    int e;
    const double m = frexp(z, &e);              // z = m * 2^e, m in [0.5, 1)
    const double y0 = static_cast<double>(__log2f(static_cast<float>(m)));
    const double y = y0 + (m * exp2_small(-y0) - 1.0) * 1.44269504088896340736;
    return static_cast<double>(e) + y;
}

// float64 scalars of the row whose pending levels are being applied (LDS; thread 0 writes, all read).
struct PendScalars {
    double lse2_q, lse2_p, tok2_q, tok2_p;   // statistics of the raw row pair
    double log2nu;                           // block ratio in front of the row (under the modified rows before it)
    double sumN, tok_adj;                    // so far: sum of the levels' log2 N; what they did to log2 q[token]
    double C;                                // constant of the current pass
    float ref_q, rc_hi, rc_nk;               // reference exponent of the target weights; the constant split as in RatioConst
};

// Constant of a pass whose ratio starts from 2^log2r: log2 (r Z_p / Z_q) minus the levels' log2 N so far.
__device__ __noinline__ void pend_pass_begin(PendScalars &row, double log2r)
{
    // (as RatioConst, with the small exponential: the library routine would claim registers that hold row data)
    row.C = row.lse2_p - row.lse2_q + log2r - row.sumN;
    row.rc_hi = static_cast<float>(row.C);
    const double kappa = exp2_small(static_cast<double>(row.rc_hi) - row.C);
    row.rc_nk = (kappa > 0.5 && kappa < 2.0) ? -static_cast<float>(kappa) : -1.0f;
}

// A level's pass is summed (S, relative to 2^ref_q): its normaliser, the drafted token's factor, the table entry
// for the passes after it, and the level's ratio moved along this row's token under the distribution it modifies.
__device__ __noinline__ PendRow pend_pass_level(PendScalars &row, PendTable &tab, double &log2mu_l, double S, int K)
{
    PendRow out;
    out.log2mu = log2mu_l; out.log2N = 0.0; out.tokadj = 0.0; out.flag = 0; out.pad = 0;
    const double W = S * exp2_small(static_cast<double>(row.ref_q) - row.lse2_q - row.sumN);   // mass of q^(l) t^K
    const double tq_eff = row.tok2_q - row.lse2_q + row.tok_adj, tp = row.tok2_p - row.lse2_p;
    log2mu_l = out.log2mu + tq_eff - tp;
    if (W > 0.0) {                               // otherwise every weight is zero and the row stays q^(l)
        out.flag = 1;
        out.log2N = log2_cheap(W);
        const double t = 1.0 - exp2_small(tp - tq_eff - out.log2mu);
        out.tokadj = t > 0.0 ? static_cast<double>(K) * log2_cheap(t) : -INFINITY;
        tab.C_hi[tab.n] = row.rc_hi; tab.neg_kappa[tab.n] = row.rc_nk;
        tab.n += 1;
        row.sumN += out.log2N;
        row.tok_adj += out.tokadj - out.log2N;
    }
    return out;
}

// The Eq. (hik) sum of a modified row from its pass (S relative to 2^ref_q).
__device__ __noinline__ double pend_pass_sum(const PendScalars &row, double S)
{
    return S * exp2_small(static_cast<double>(row.ref_q) - row.lse2_q - row.sumN);
}

// Pending modifications as the chain kernel sees them (nlev = 0: none).
constexpr int kRow0Threads = 256;

// Partial statistics of the rows 0 that the K drafts of a prefix share (position 0 of every draft is
// conditioned on the prefix alone; Algorithm 3).  grid (kRow0Parts, batch, 2): workgroup (i, b, m) reduces
// slice i of row 0 of draft 0 of prefix b, in the target (m = 0) or draft (m = 1) tensor, to
// sum_x 2^(c z[x] - ref) with an integral reference exponent, so that the slices combine exactly.
// The tokens the K drafts start with are left out of the float32 sums of the slice they fall in (leave_out); the
// first wave adds the weight of each distinct one in float64.
template <typename T>
__global__ void __launch_bounds__(kRow0Threads)
k_row0_parts(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens, int K, int L,
             int V, float c, Row0Part *__restrict__ parts)
{
    static_assert(kMaxDrafts <= kWave, "one lane of the first wave per draft");
    __shared__ double sh_d[kRow0Threads / kWave];
    __shared__ float sh_f[kRow0Threads / kWave];
    __shared__ int sh_tok[kMaxDrafts];                     // the distinct first tokens that fall into this slice
    __shared__ int sh_ntok;
    const int part = blockIdx.x, b = blockIdx.y, m = blockIdx.z;
    const long long bk0 = static_cast<long long>(b) * K;
    const T *row = m ? draft + bk0 * L * static_cast<long long>(V) : target + bk0 * (L + 1) * static_cast<long long>(V);
    constexpr int PV = Elem<T>::kPerVec;
    const int nvec = V / PV;
    const int per = (nvec + kRow0Parts - 1) / kRow0Parts;
    const int lo = part * per, hi = lo + per < nvec ? lo + per : nvec;
    // four loads in flight per thread; the first four are issued before the list of tokens is made
    auto load4 = [&](int i, U4 (&v)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = i + j * kRow0Threads;
            v[j] = load16_stream(row + static_cast<long long>(idx < hi ? idx : i) * PV);
        }
    };
    U4 v[4];
    int i = lo + static_cast<int>(threadIdx.x);
    if (i < hi) load4(i, v);
    double tok2_mine = -static_cast<double>(__builtin_inff());     // first wave: scaled logit of the lane's token, if it is listed
    if (threadIdx.x < kWave) {
        const int j = threadIdx.x;
        int tok = j < K ? tokens[(bk0 + j) * L] : 0;
        tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
        bool keep = j < K && tok / PV >= lo && tok / PV < hi;
        for (int e = 0; e < K; ++e) {                          // not a token an earlier draft has too
            const int other = __builtin_amdgcn_readlane(tok, e);
            if (e < j && other == tok) keep = false;
        }
        const unsigned long long kept = __ballot(keep);
        if (keep) {
            sh_tok[__popcll(kept & ((1ull << j) - 1ull))] = tok;
            tok2_mine = static_cast<double>(Elem<T>::scalar(row + tok)) * static_cast<double>(c);
        }
        if (j == 0) sh_ntok = __popcll(kept);
    }
    __syncthreads();
    const int ntok = __builtin_amdgcn_readfirstlane(sh_ntok);
    auto drop = [&](float (&z)[PV], int idx) {
        for (int e = 0; e < ntok; ++e) {
            const int tok = sh_tok[e];
            leave_out(z, idx == tok / PV, tok % PV);
        }
    };
    RunningSum acc;
    while (i < hi) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i + j * kRow0Threads < hi) {
                float z[PV];
                Elem<T>::unpack(v[j], z);
                drop(z, i + j * kRow0Threads);
                acc.add(z, c);
            }
        }
        i += 4 * kRow0Threads;
        if (i < hi) load4(i, v);
    }
    const float M = block_max(acc.m2, sh_f);
    const double mine = static_cast<double>(acc.Z) * exp2(static_cast<double>(acc.m2) - static_cast<double>(M));
    const double total = block_sum(acc.Z > 0.0f ? mine : 0.0, sh_d);
    if (threadIdx.x < kWave) {                                 // (uniform over the first wave)
        // the listed tokens' weights, relative to the largest of them
        double tmax = tok2_mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) tmax = fmax(tmax, __shfl_xor(tmax, o));
        const double wsum = wave_sum(tok2_mine > -1.0e300 ? exp2(tok2_mine - tmax) : 0.0);
        if (threadIdx.x == 0) {
            double ref = static_cast<double>(M), Z = total;
            if (tmax > -1.0e300) {                             // (-inf: none listed, or all of them masked entries)
                ref = fmax(ref, tmax);
                Z = (total > 0.0 ? total * exp2(static_cast<double>(M) - ref) : 0.0) + wsum * exp2(tmax - ref);
            }
            Row0Part out;
            out.ref = floor(ref);
            out.Z = Z * exp2(ref - out.ref);
            parts[(static_cast<long long>(b) * 2 + m) * kRow0Parts + part] = out;
        }
    }
}

__device__ __forceinline__ double lane_d(double v, int lane)
{
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane(static_cast<int>(bits), lane);
    const int hi = __builtin_amdgcn_readlane(static_cast<int>(bits >> 32), lane);
    return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned>(lo));
}

// Position 0 of chain bk when the prefix's drafts share their rows 0: the row statistics from the slices'
// partial sums (lanes 0..15 of every wave take the target slices, lanes 16..31 the draft slices; the same
// butterfly in every workgroup, so every draft of the prefix gets the same bits), the chain's own token
// read from draft 0's rows.  Every wave computes the same values; thread 0 stores the RowStat.  Returns the
// log2 block ratio after that token (and in log2P the log2 of the token's draft probability).
template <typename T>
__device__ __forceinline__ double row0_from_parts(const Row0Part *parts, const T *target, const T *draft,
                                                  const int32_t *tokens, long long bk, int K, int L, int V, float c,
                                                  double c_rel, RowStat *stats, double &log2P)
{
    static_assert(kRow0Parts == 16, "one 16-lane row per tensor");
    const long long b = bk / K;
    const int lane = threadIdx.x & 31;
    const Row0Part pt = parts[b * 2 * kRow0Parts + lane];
    const bool live = pt.Z > 0.0;
    double ref = live ? pt.ref : -1.0e300;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) ref = fmax(ref, __shfl_xor(ref, o));
    const double d = pt.ref - ref;                            // an integer <= 0
    double Z = (live && d > -2000.0) ? ldexp(pt.Z, static_cast<int>(d)) : 0.0;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) Z += __shfl_xor(Z, o);
    const double lse2 = ref + log2_refined(Z);
    int tok = tokens[bk * L];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    const long long bk0 = b * K;
    RowStat st;
    st.lse2_q = lane_d(lse2, 0); st.lse2_p = lane_d(lse2, 16);
    st.tok2_q = token_scaled(static_cast<double>(Elem<T>::scalar(target + bk0 * (L + 1) * static_cast<long long>(V) + tok)) * static_cast<double>(c), st.lse2_q, c_rel);
    st.tok2_p = token_scaled(static_cast<double>(Elem<T>::scalar(draft + bk0 * L * static_cast<long long>(V) + tok)) * static_cast<double>(c), st.lse2_p, c_rel);
    if (threadIdx.x == 0) stats[bk * L] = st;
    log2P = st.tok2_p - st.lse2_p;
    return (st.tok2_q - st.lse2_q) - (st.tok2_p - st.lse2_p);
}

struct ChainPend {
    const double *carry;       // [nlev][batch]
    const int32_t *count;      // [nlev][batch]
    PendRow *rows;             // [nlev][batch * K * L], written for the final-token kernel
    int nlev, batch;
};

// sum over this thread's on-chip vectors of the row pair of the weights w (ot_weights, or pending_weights
// when tab holds levels), relative to 2^shift_q.  Register slots are all full (the host picks RS so).
template <typename T, int RS, int... Js>
__device__ __forceinline__ float onchip_sum(std::integer_sequence<int, Js...>, U4 (&rq)[RS], U4 (&rp)[RS],
                                            const LdsSlots &lds, unsigned tid, int rem, int n_on, float c, float shift_q,
                                            const PendTable &tab, const RatioConst &rc, int K)
{
    constexpr int PV = Elem<T>::kPerVec;
    float acc = 0.0f;
    const bool plain = tab.n == 0;
    // Four entries at a time and one slot strictly after the other (the opaque touch of the accumulator keeps
    // the compiler from interleaving slots): the slots themselves occupy most of the register file.
    auto one = [&](const U4 &q, const U4 &p) {
        float zq[PV], zp[PV], wq[PV], w[PV];
        Elem<T>::unpack(q, zq);
        Elem<T>::unpack(p, zp);
        if (plain) ot_weights(zq, zp, c, shift_q, rc, K, wq, w);
        else pending_weights(zq, zp, c, shift_q, tab, rc, K, wq, w);
        float a = 0.0f;
#pragma unroll
        for (int j = 0; j < PV; ++j) a += w[j];
        acc += a;
        asm volatile("" : "+v"(acc));
    };
    // Register slots one strictly after the other: the opaque touch makes a slot's registers (and the running
    // sum) pass through a point in program order, so that no slot's unpacked values are formed ahead of time.
    auto reg = [&](U4 &q, U4 &p) {
        asm volatile("" : "+v"(q.x), "+v"(q.y), "+v"(q.z), "+v"(q.w), "+v"(acc));
        asm volatile("" : "+v"(p.x), "+v"(p.y), "+v"(p.z), "+v"(p.w), "+v"(acc));
        one(q, p);
    };
    (reg(rq[Js], rp[Js]), ...);
    for (int s = 0; s < kLdsSlots; ++s) {
        const int J = RS + s;
        if (J < n_on && J * kChainThreads < rem) one(lds_vec(lds, s, 0, tid), lds_vec(lds, s, 1, tid));
    }
    return acc;
}

template <typename T, int KP, int RS, bool PEND>
__global__ void __launch_bounds__(kChainThreads)
k_chain(const T *__restrict__ target, const T *__restrict__ draft, const int32_t *__restrict__ tokens,
        int K, int L, int V, long long nchains, float c, RowStat *__restrict__ stats, double *__restrict__ s_out,
        double *__restrict__ e_out,
        int32_t *__restrict__ final_counter, ChainPend pend, int first_row, const Row0Part *__restrict__ row0, double c_rel,
        int32_t *__restrict__ later, int later_stride)
{
    __shared__ U4 lds_all[kLdsSlots * 2 * kChainThreads];
    __shared__ double sh_d[3 * kChainWaves];
    __shared__ double sh_sumrow[2][2];                     // log2 of the block ratio and of the drafts' joint probability in front
                                                           // of the row in sweep 2: written by thread 0 when the row's statistics
                                                           // are known, in the entry of the iteration's parity, read one iteration later
    __shared__ int sh_nlater;                              // rows handed to k_chain_excess so far (the summing thread only)
    __shared__ TokenTerm sh_tokterm[2];                    // the drafted token of the row in sweep 2 (written and read like sh_sumrow)
    __shared__ PendTable sh_tab;                           // PEND only: levels that modify the current row
    __shared__ double sh_mu[kMaxPend];                     //            log2 block ratio of every level in front of the current row
    __shared__ int sh_cnt[kMaxPend];                       //            rows every level modifies (this prefix)
    __shared__ PendScalars sh_row;                         //            float64 scalars of the current row
    __shared__ ChainPend sh_pend;                          //            the kernel argument, kept out of the scalar registers
    __shared__ int sh_sum_done;                            //            the row in sweep 2 already has its sum (modified row)
    if constexpr (PEND) {
        if (threadIdx.x == 0) { sh_pend = pend; sh_sum_done = 0; }
        __syncthreads();
    }

    // The thread that finishes a row's Eq. (hik) sum is the second wave's first: thread 0 stores the statistics of the
    // row being loaded in the same iteration, and the two pieces of scalar work then run side by side.
    constexpr unsigned kSumThread = kWave;
    if (threadIdx.x == kSumThread) sh_nlater = 0;
    constexpr int PV = Elem<T>::kPerVec;
    constexpr int NS = RS + kLdsSlots;                     // slots kept on chip
    const unsigned tid = threadIdx.x;
    const unsigned lds_wave_addr = static_cast<unsigned>(
        reinterpret_cast<uintptr_t>(static_cast<void *>(&lds_all[tid & ~(kWave - 1u)])));
    const LdsSlots lds{lds_all, static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(lds_wave_addr)))};
    const int nvec = V / PV;                               // host guarantees nvec >= RS * 512
    const int rem = nvec - static_cast<int>(tid);          // slot j holds a vector of this thread iff j*512 < rem
    const int nslots = (nvec + kChainThreads - 1) / kChainThreads;
    const int n_on = nslots < NS ? nslots : NS;            // on-chip slots in use
    // This workgroup walks the (prefix, draft) chains blockIdx.x, blockIdx.x + gridDim.x, ... one after
    // the other as ONE sequence of rows: the last sum of a chain overlaps the first loads of the next.
    // (32-bit arithmetic: the host checks that batch * K * (L + 1) stays below 2^31)
    const int nmine = static_cast<int>((nchains - blockIdx.x + gridDim.x - 1) / gridDim.x);
    // first_row = 1: the prefix's drafts share their rows 0, whose statistics come from k_row0_parts, and a
    // chain is its rows 1 .. L-1 (the host guarantees L >= 2 then)
    const int rpc = L - first_row;                         // rows per chain
    const int nrows = nmine * rpc;                         // rows of this workgroup, in the order it visits them
    auto chain_of = [&](int g) { return static_cast<long long>(blockIdx.x) + static_cast<long long>(g / rpc) * gridDim.x; };

    U4 rq[RS], rp[RS];
#pragma unroll
    for (int j = 0; j < RS; ++j) { rq[j] = U4{0, 0, 0, 0}; rp[j] = U4{0, 0, 0, 0}; }

    RowConsts rc_sum;                                      // constants of the row in sweep 2
    rc_sum.c = c; rc_sum.K = K; rc_sum.nref_q = rc_sum.nref_p = 0.0f; rc_sum.C2_hi = 0.0f; rc_sum.neg_kappa = -1.0f;
    double Zq_prev = 1.0;                                  // target normaliser of the row in sweep 2
    double log2nu = 0.0;                                   // block ratio of the rows before the row being loaded
    double log2P = 0.0;                                    // joint draft probability of their tokens

    // Iteration g overlaps three things slot by slot: sweep 2 of row g-1 (its Eq. (hik) sum, unless it
    // is the first row of its chain), the load of row g into the slot that sweep 2 just released, and
    // sweep 1 of row g on the slot loaded kLag steps earlier.  Loads are therefore issued evenly over
    // the whole row period and the memory pipeline never drains between rows.
    // The drafted token's two logits (the reference exponents of a row's first sweep) are fetched one row ahead, as
    // loaded: the wait for them then falls at the end of the previous iteration, where no other load is in flight,
    // and not behind the first LDS fills of their own row, which it would drain.  The fetch brings the whole 16-byte
    // vector the token lies in, one element per lane: lanes 0 .. PV-1 of every wave the target row's, lanes
    // PV .. 2PV-1 the draft row's (the lanes above repeat them).  That vector's weights are summed apart from the
    // sweep (sweep1_vec's `leave_out`), the token's own in float64.
    const unsigned lane = tid & (kWave - 1u);
    const bool lane_p = (lane / PV) & 1u;                  // this lane's element of the token vector is the draft row's
    auto token_vector = [&](int gg, uint32_t &bits, int &tok_out) {
        const int gc = gg < nrows ? gg : nrows - 1;        // keeps every address in bounds
        const long long bk = chain_of(gc);
        const int r = first_row + gc % rpc;
        int tok = tokens[bk * L + r];
        tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
        tok_out = tok;
        const long long at = static_cast<long long>(tok / PV) * PV + (lane % PV);      // < V: V is a multiple of PV
        const T *row = lane_p ? draft + (bk * L + r) * static_cast<long long>(V)
                              : target + (bk * (L + 1) + r) * static_cast<long long>(V);
        bits = Elem<T>::bits(row + at);
    };
    uint32_t tokvec_next = 0;
    int tok_next = 0;
    if (nrows > 0) token_vector(0, tokvec_next, tok_next);
    for (int g = 0; g <= nrows; ++g) {
        const bool do_new = g < nrows;                     // a row is being loaded and gets its statistics
        const int g_new = do_new ? g : nrows - 1;          // keeps every address in bounds
        const long long bk_new = chain_of(g_new);
        const int r_new = first_row + g_new % rpc;
        const int g_old = g >= 1 ? g - 1 : 0;
        const long long bk_old = chain_of(g_old);
        const int r_old = first_row + g_old % rpc;
        bool do_sum = g >= 1 && r_old >= 1;                // rows >= 1 get their Eq. (hik) sum
        // (written by thread 0 before the barrier that ends the previous row's level passes, and not again before
        // the barriers of this iteration's row-end reduction, which every wave passes after this read)
        if constexpr (PEND) do_sum = do_sum && __builtin_amdgcn_readfirstlane(sh_sum_done) == 0;
        const T *qnew = target + (bk_new * (L + 1) + r_new) * static_cast<long long>(V);
        const T *pnew = draft + (bk_new * L + r_new) * static_cast<long long>(V);
        const T *qold = target + (bk_old * (L + 1) + r_old) * static_cast<long long>(V);
        const T *pold = draft + (bk_old * L + r_old) * static_cast<long long>(V);
        const unsigned off_new = do_new ? tid * 16u : 0u;  // after the last row: one harmless line
        if (do_new && r_new == first_row && tid == 0 && bk_new % K == 0)
            final_counter[bk_new / K] = 0;                 // arrival counter of the final-token kernel

        // Reference exponents of the new row: its token's logits (the drafted token was
        // sampled from this draft row, so no entry can exceed it by a factor near 2^127
        // unless the row is extremely peaked; that case is caught below).
        const int tok_new = __builtin_amdgcn_readfirstlane(tok_next);
        const uint32_t tokvec = tokvec_next;
        const float zq_tok = Elem<T>::from_bits(__builtin_amdgcn_readlane(tokvec, tok_new % PV));
        const float zp_tok = Elem<T>::from_bits(__builtin_amdgcn_readlane(tokvec, PV + tok_new % PV));
        if (do_new) token_vector(g + 1, tokvec_next, tok_next);      // (the last row's again after the last row)
        RowConsts rc_new;
        rc_new.c = c; rc_new.K = K; rc_new.C2_hi = 0.0f; rc_new.neg_kappa = -1.0f;
        rc_new.nref_q = -(zq_tok * c); rc_new.nref_p = -(zp_tok * c);
        // weights of the token's neighbours in its vector (every wave computes the same two sums)
        float nb_q, nb_p;
        {
            const float w = exp2_fast(fmaf(Elem<T>::from_bits(tokvec), c, lane_p ? rc_new.nref_p : rc_new.nref_q));
            const bool nb = lane < 2u * PV && lane % PV != static_cast<unsigned>(tok_new % PV);
            nb_q = wave_sum_f32(nb && !lane_p ? w : 0.0f);
            nb_p = wave_sum_f32(nb && lane_p ? w : 0.0f);
        }

        float Zq = 0.0f, Zp = 0.0f, acc = 0.0f;
        StepCtx<T> cx{qnew, pnew, rc_sum, rc_new, tid, off_new, nvec, rem, n_on, do_new, do_sum,
                      (tok_new / PV) / kChainThreads, tid == static_cast<unsigned>((tok_new / PV) % kChainThreads)};
        run_steps<T, KP, RS>(std::make_integer_sequence<int, NS + kLag>{}, cx, rq, rp, lds, Zq, Zp, acc);
        // vectors that do not fit on chip: read for the statistics now, once more for the sum; the
        // loads of the next slot are issued before the arithmetic of the current one
        if (NS < nslots) {
            const U4 zero{0, 0, 0, 0};
            auto fetch = [&](int j, U4 &a, U4 &b, U4 &cc, U4 &dd) {
                const bool live = j < nslots && j * kChainThreads < rem;
                a = (live && do_new) ? load_slot(qnew, j, tid) : zero;
                b = (live && do_new) ? load_slot(pnew, j, tid) : zero;
                cc = (live && do_sum) ? load_slot(qold, j, tid) : zero;
                dd = (live && do_sum) ? load_slot(pold, j, tid) : zero;
            };
            U4 a0, b0, c0, d0;
            fetch(NS, a0, b0, c0, d0);
            for (int j = NS; j < nslots; ++j) {
                U4 a1, b1, c1, d1;
                fetch(j + 1, a1, b1, c1, d1);
                if (j * kChainThreads < rem) {
                    if (do_new) sweep1_vec<T>(a0, b0, rc_new, Zq, Zp, j == cx.tok_slot, cx.tok_mine);
                    if (do_sum) sweep2_vec<T, KP>(c0, d0, rc_sum, acc);
                }
                a0 = a1; b0 = b1; c0 = c1; d0 = d1;
            }
        }

        asm volatile("" : "+v"(tokvec_next));              // the next row's token vector has arrived by here
        double Zq_tot = static_cast<double>(Zq), Zp_tot = static_cast<double>(Zp), s_tot = static_cast<double>(acc);
        block_sum3(Zq_tot, Zp_tot, s_tot, sh_d);
        Zq_tot = uniform_d(Zq_tot); Zp_tot = uniform_d(Zp_tot); s_tot = uniform_d(s_tot);
        // The token's own weight is 2^(what the rounding of its reference exponent to float32 left over), within
        // 1e-5 of one: three terms of the exponential series, in float64.  The sums so far hold everything else, so
        // a row whose mass sits on its drafted token keeps the rest to float32 RELATIVE accuracy.
        {
            const double xq = fma(static_cast<double>(zq_tok), static_cast<double>(c), static_cast<double>(rc_new.nref_q)) *
                              0.69314718055994530942;
            const double xp = fma(static_cast<double>(zp_tok), static_cast<double>(c), static_cast<double>(rc_new.nref_p)) *
                              0.69314718055994530942;
            Zq_tot += static_cast<double>(nb_q) + (1.0 + xq + 0.5 * xq * xq);
            Zp_tot += static_cast<double>(nb_p) + (1.0 + xp + 0.5 * xp * xp);
        }
        if (do_sum && tid == kSumThread) {
            const double inv_Zq = 1.0 / Zq_prev;
            double s_val = s_tot * inv_Zq;
            // The drafted token's own term once more in float64 where its p/(nu q) is near one: formed from a float32
            // exponential, 1 - p/(nu q) is good to 6e-8 absolute only, and on a row whose mass sits on its drafted
            // token, in front of a block ratio near one, that term is a good part of the whole sum.  The sweep's
            // value of the term is taken out again (the same operations give the same bits).
            {
                const TokenTerm *tt = &sh_tokterm[(g - 1) & 1];
                const float zq = tt->zq, zp = tt->zp;
                const float u = fmaf(exp2_fast(fmaf(zp - zq, c, -rc_sum.C2_hi)), rc_sum.neg_kappa, 1.0f);
                if (fabsf(u) < kTokenTermBelow) {
                    float t1[1] = {__builtin_amdgcn_fmed3f(u, 0.0f, 1.0f)};
                    pow_inplace<KP>(t1, K);
                    s_val = token_term_call(s_tot, exp2_fast(fmaf(zq, c, rc_sum.nref_q)) * t1[0], inv_Zq, tt, K);
                }
            }
            s_out[bk_old * L + r_old] = s_val;
            // where s and g = (1 - 1/nu)^K nearly cancel, Eq. (hik) needs nu^2 (s - g) summed term by term (rare:
            // peaked rows, large block ratios).  The row has left the chip by now, and one workgroup reading it again
            // alone would hold up the whole grid for the time of a row: it is marked, and k_chain_excess, launched
            // behind this kernel, spreads the marked rows over the chip.
            bool again = false;
            if constexpr (!PEND) {
                const double *front = sh_sumrow[(g - 1) & 1];
                if (excess_wanted(static_cast<float>(front[0]), static_cast<float>(s_val), K) && sh_nlater + 1 < later_stride &&
                    excess_needed_call(front[0], front[1], s_val, K)) {
                    again = true;
                    sh_nlater = sh_nlater + 1;
                    later[static_cast<size_t>(blockIdx.x) * later_stride + sh_nlater] = static_cast<int32_t>(bk_old * L + r_old);
                }
            }
            e_out[bk_old * L + r_old] = again ? kExcessPending : -1.0;
        }
        if (do_new) {
            if (r_new == first_row) {                      // a new chain starts from the empty block ...
                log2nu = 0.0; log2P = 0.0;
                if (first_row) {                           // ... or from its token at the shared position 0
                    log2nu = uniform_d(row0_from_parts<T>(row0, target, draft, tokens, bk_new, K, L, V, c, c_rel, stats, log2P));
                    log2P = uniform_d(log2P);
                }
            }
            float ref_q = -rc_new.nref_q, ref_p = -rc_new.nref_p;
            // A sum far above 1 means that the entries that matter lie far above the token's logit: their
            // exponents, formed in float32, then carry an absolute error of half an ulp of a large number
            // (3.8e-6 at 2^6), which a row dominated by one entry passes on to its log-normaliser in full.
            // Beyond 2^30 (a drafted token of probability below 1e-9, or float32 overflow) the row is
            // summed again with its exact maximum as reference.
            if (!(Zq_tot < kTokenRefLimit) || !(Zq_tot > 0.0)) {
                const ExactStats e = exact_row_stats<T>(qnew, nvec, c, sh_d);
                ref_q = e.ref; Zq_tot = e.Z;
            }
            if (!(Zp_tot < kTokenRefLimit) || !(Zp_tot > 0.0)) {
                const ExactStats e = exact_row_stats<T>(pnew, nvec, c, sh_d);
                ref_p = e.ref; Zp_tot = e.Z;
            }
            // both logarithms in one go: even lanes take the target's sum, odd lanes the draft's
            const double lg = log2_refined((tid & 1) ? Zp_tot : Zq_tot);
            const double lse2_q = static_cast<double>(ref_q) + lane_d(lg, 0);
            const double lse2_p = static_cast<double>(ref_p) + lane_d(lg, 1);
            const double tok2_q = token_scaled(static_cast<double>(zq_tok) * static_cast<double>(c), lse2_q, c_rel);
            const double tok2_p = token_scaled(static_cast<double>(zp_tok) * static_cast<double>(c), lse2_p, c_rel);
            if (tid == 0) {
                RowStat st;
                st.lse2_q = lse2_q; st.lse2_p = lse2_p; st.tok2_q = tok2_q; st.tok2_p = tok2_p;
                stats[bk_new * L + r_new] = st;
            }
            double tok_adj = 0.0;                          // what the pending levels do to log2 q[token] of this row
            if constexpr (PEND) {
                // All float64 work of the levels is done by thread 0 in a function of its own (values travel through
                // LDS): the other threads only sweep their on-chip vectors, so the register slots need not be spilled.
                const int b = static_cast<int>(bk_new / K);
                const int nlev_u = __builtin_amdgcn_readfirstlane(sh_pend.nlev);
                const long long n_rows = static_cast<long long>(sh_pend.batch) * K * L, pair = bk_new * L + r_new;
                __syncthreads();
                if (r_new == 0 && tid < static_cast<unsigned>(nlev_u)) {
                    sh_mu[tid] = sh_pend.carry[static_cast<size_t>(tid) * sh_pend.batch + b] * 1.44269504088896340736;
                    sh_cnt[tid] = sh_pend.count[static_cast<size_t>(tid) * sh_pend.batch + b];
                }
                if (tid == 0) {
                    sh_tab.n = 0;
                    sh_row.lse2_q = lse2_q; sh_row.lse2_p = lse2_p; sh_row.tok2_q = tok2_q; sh_row.tok2_p = tok2_p;
                    sh_row.log2nu = log2nu; sh_row.sumN = 0.0; sh_row.tok_adj = 0.0; sh_row.ref_q = ref_q;
                }
                __syncthreads();
                for (int l = 0; l <= nlev_u; ++l) {     // uniform; pass nlev is the row's Eq. (hik) sum against the modified row
                    const bool is_sum = l == nlev_u;
                    const bool live = is_sum ? (sh_tab.n > 0 && r_new >= 1) : (r_new < sh_cnt[l]);
                    if (live) {
                        if (tid == 0) pend_pass_begin(sh_row, is_sum ? sh_row.log2nu : sh_mu[l]);
                        __syncthreads();
                        RatioConst rc(0.0);
                        rc.C2_hi = sh_row.rc_hi; rc.neg_kappa = sh_row.rc_nk;
                        double S = static_cast<double>(onchip_sum<T, RS>(std::make_integer_sequence<int, RS>{}, rq, rp, lds, tid, rem,
                                                                         n_on, c, ref_q, sh_tab, rc, K));
                        double unused = 0.0;
                        block_sum2(S, unused, sh_d);
                        if (tid == 0) {
                            if (is_sum) { s_out[pair] = pend_pass_sum(sh_row, S); e_out[pair] = -1.0; }
                            else sh_pend.rows[l * n_rows + pair] = pend_pass_level(sh_row, sh_tab, sh_mu[l], S, K);
                        }
                        __syncthreads();
                    } else if (!is_sum && tid == 0) {
                        PendRow out;
                        out.log2mu = 0.0; out.log2N = 0.0; out.tokadj = 0.0; out.flag = 0; out.pad = 0;
                        sh_pend.rows[l * n_rows + pair] = out;
                    }
                }
                // a modified row has its sum (or needs none: row 0); thread 0 is the only writer of sh_tab.n, which is
                // final here, and the barrier below publishes the flag before any wave starts the next row
                if (tid == 0) sh_sum_done = sh_tab.n > 0;
                __syncthreads();
                tok_adj = sh_row.tok_adj;
            }
            // constants of this row's sweep 2 (next iteration)
            const double C2 = lse2_p - lse2_q + log2nu;
            const double C2s = ratio_const(lse2_p, lse2_q, log2nu, c_rel);    // as the sweep takes it
            rc_sum.nref_q = -ref_q;
            rc_sum.C2_hi = static_cast<float>(C2s);
            const double dk = (static_cast<double>(rc_sum.C2_hi) - C2s) * 0.693147180559945309417;
            rc_sum.neg_kappa = (dk > -0.25 && dk < 0.25) ? -static_cast<float>(1.0 + dk + 0.5 * dk * dk) : -1.0f;
            Zq_prev = uniform_d(Zq_tot);
            if (tid == 0) {
                sh_sumrow[g & 1][0] = log2nu; sh_sumrow[g & 1][1] = log2P;
                TokenTerm tt;
                tt.zq = zq_tok; tt.zp = zp_tok; tt.log2q = tok2_q - lse2_q; tt.log2r = (tok2_p - tok2_q) - C2;
                sh_tokterm[g & 1] = tt;
            }
            log2nu = uniform_d(log2nu + ((tok2_q - lse2_q + tok_adj) - (tok2_p - lse2_p)));
            log2P = uniform_d(log2P + (tok2_p - lse2_p));
        }
    }
    if constexpr (!PEND)
        if (tid == kSumThread) later[static_cast<size_t>(blockIdx.x) * later_stride] = sh_nlater;   // (every workgroup, also when it is 0)
}

// E = nu^2 (s - g) of the rows k_chain handed over, straight from memory, in kPendParts parts per row which the
// decision kernel adds up in part order.  Every workgroup reads the lengths of all `nlists` lists (nearly always all
// 0: it leaves at once), numbers the listed rows in list order and takes the units blockIdx.x, blockIdx.x +
// gridDim.x, ... of (row, part), part fastest.  Every wave fetches the statistics of the row's chain itself, one row
// per lane (L <= 62).
template <typename T>
__global__ void __launch_bounds__(kExcessThreads)
k_chain_excess(const T *__restrict__ target, const T *__restrict__ draft, int K, int L, int V, float c,
               const RowStat *__restrict__ stats, const int32_t *__restrict__ later, int nlists, int later_stride,
               double *__restrict__ e_part)
{
    constexpr int kPer = kMaxChainGrid / kExcessThreads;   // lists per thread
    __shared__ double sh_d[kExcessThreads / kWave];
    __shared__ int sh_before[kMaxChainGrid + 1];           // rows in the lists before list w; entry nlists: all of them
    __shared__ int sh_wave[kExcessThreads / kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wid = tid / kWave;
    int cnt[kPer], mine = 0;
#pragma unroll
    for (int a = 0; a < kPer; ++a) {
        const int w = tid * kPer + a;
        const int n = w < nlists ? later[static_cast<size_t>(w) * later_stride] : 0;
        cnt[a] = n < 0 ? 0 : (n > later_stride - 1 ? later_stride - 1 : n);
        mine += cnt[a];
    }
    if (__syncthreads_or(mine) == 0) return;               // no row anywhere
    int incl = mine;                                       // inclusive scan over the wave, then over the waves
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) sh_wave[wid] = incl;
    __syncthreads();
    int before = incl - mine;
    for (int v = 0; v < wid; ++v) before += sh_wave[v];
#pragma unroll
    for (int a = 0; a < kPer; ++a) {
        sh_before[tid * kPer + a] = before;
        before += cnt[a];
    }
    if (tid == kExcessThreads - 1) sh_before[kMaxChainGrid] = before;
    __syncthreads();
    const int nrows = sh_before[kMaxChainGrid];
    constexpr int PV = Elem<T>::kPerVec;
    constexpr int kAhead = 4;                              // vector pairs in flight per thread
    const int nvec = V / PV;
    const int per = (nvec + kPendParts - 1) / kPendParts;
    for (long long u = blockIdx.x; u < static_cast<long long>(nrows) * kPendParts; u += gridDim.x) {      // uniform
        const int r = static_cast<int>(u / kPendParts), part = static_cast<int>(u % kPendParts);
        int w = 0;                                         // the list that holds row r: the last one with sh_before[w] <= r
        for (int step = kMaxChainGrid / 2; step >= 1; step >>= 1)
            if (w + step < kMaxChainGrid && sh_before[w + step] <= r) w += step;
        const long long pair = later[static_cast<size_t>(w) * later_stride + 1 + (r - sh_before[w])];
        const long long bk = pair / L;
        const int i = static_cast<int>(pair % L);
        const int lo = part * per, hi = lo + per < nvec ? lo + per : nvec;
        const T *qrow = target + (bk * (L + 1) + i) * static_cast<long long>(V);
        const T *prow = draft + pair * static_cast<long long>(V);
        // the first vectors (nearly always all of the part's) are asked for before the row's constants are made: the
        // statistics' latency and their float64 arithmetic pass while the vectors travel
        U4 q[kAhead], pp[kAhead];
        const int last = hi > lo ? hi - 1 : nvec - 1;      // what a lane past the part's end reads again (inside the row)
        auto fetch = [&](int v0) {
#pragma unroll
            for (int a = 0; a < kAhead; ++a) {
                const int v = v0 + a * kExcessThreads;
                const long long at = static_cast<long long>(v < hi ? v : last) * PV;
                q[a] = load16_stream(qrow + at);
                pp[a] = load16_stream(prow + at);
            }
        };
        const RowStat st = stats[bk * L + (lane < L ? lane : L - 1)];
        fetch(lo + tid);
        const double ratio = (st.tok2_q - st.lse2_q) - (st.tok2_p - st.lse2_p);   // log2 of the row's token ratio
        double log2nu = 0.0;                               // added up as k_chain does: the same bits
        for (int j = 0; j < i; ++j) log2nu += lane_d(ratio, j);
        const ExcessConst ec = make_excess_const(lane_d(st.lse2_q, i), lane_d(st.lse2_p, i), log2nu, K, c);
        float acc = 0.0f;
        for (int v0 = lo + tid; v0 < hi; v0 += kAhead * kExcessThreads) {
#pragma unroll
            for (int a = 0; a < kAhead; ++a) {
                float zq[PV], zp[PV];
                Elem<T>::unpack(q[a], zq);
                Elem<T>::unpack(pp[a], zp);
                if (v0 + a * kExcessThreads < hi) acc += excess_terms(zq, zp, ec);
            }
            if (v0 + kAhead * kExcessThreads < hi) fetch(v0 + kAhead * kExcessThreads);
        }
        // (a part without vectors, where the row has fewer of them than parts, adds 0)
        const double e_val = block_sum(static_cast<double>(acc), sh_d) * ec.scale;
        if (tid == 0) e_part[pair * kPendParts + part] = e_val;
    }
}

// Workgroups that can be resident at once: one per compute unit (a workgroup takes 144 KiB of LDS).
int resident_workgroups()
{
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        cached[dev] = (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
        if (cached[dev] > kMaxChainGrid) cached[dev] = kMaxChainGrid;      // (the workspace holds that many row lists)
    }
    return cached[dev];
}

template <typename T, int KP, bool PEND>
hipError_t launch_kp(const Problem &p)
{
    RowStat *stats = reinterpret_cast<RowStat *>(p.ws + p.lay.stats);
    double *s = reinterpret_cast<double *>(p.ws + p.lay.s);
    const long long nchains = static_cast<long long>(p.batch) * p.K;
    const long long cus = resident_workgroups();
    const dim3 grid(static_cast<unsigned>(nchains < cus ? nchains : cus));
    const int stride = later_list_entries(nchains, grid.x, p.L);
    const T *target = static_cast<const T *>(p.target);
    const T *draft = static_cast<const T *>(p.draft);
    const int full_slots = (p.V / Elem<T>::kPerVec) / kChainThreads;
    ChainPend pend;
    pend.carry = p.pend_carry; pend.count = p.pend_count;
    pend.rows = reinterpret_cast<PendRow *>(p.ws + p.lay.pend);
    pend.nlev = PEND ? p.pend_levels : 0; pend.batch = p.batch;
    // rows 0 shared by a prefix's drafts: reduced once per prefix by a small kernel of their own
    const int first_row = (!PEND && p.shared_row0 && p.L >= 2) ? 1 : 0;
    Row0Part *row0 = reinterpret_cast<Row0Part *>(p.ws + p.lay.row0);
    if (first_row)
        hipLaunchKernelGGL((k_row0_parts<T>), dim3(kRow0Parts, static_cast<unsigned>(p.batch), 2), dim3(kRow0Threads), 0,
                           p.stream, target, draft, p.tokens, p.K, p.L, p.V, p.c, row0);
#define SPECGBV_LAUNCH(RS)                                                                                  \
    hipLaunchKernelGGL((k_chain<T, KP, RS, PEND>), grid, dim3(kChainThreads), 0, p.stream, target, draft,  \
                       p.tokens, p.K, p.L, p.V, nchains, p.c, stats, s,                                    \
                       reinterpret_cast<double *>(p.ws + p.lay.excess),                                    \
                       reinterpret_cast<int32_t *>(p.ws + p.lay.counter), pend, first_row, row0, p.c_rel,     \
                       reinterpret_cast<int32_t *>(p.ws + p.lay.later), stride)
    if (full_slots >= 23) SPECGBV_LAUNCH(23);
    else if (full_slots >= 15) SPECGBV_LAUNCH(15);
    else SPECGBV_LAUNCH(7);
#undef SPECGBV_LAUNCH
    return hipGetLastError();
}

template <typename T>
hipError_t launch_excess_typed(const Problem &p)
{
    const long long nchains = static_cast<long long>(p.batch) * p.K;
    const long long cus = resident_workgroups();
    const long long grid = nchains < cus ? nchains : cus;                  // k_chain's grid: one list per workgroup
    hipLaunchKernelGGL((k_chain_excess<T>), dim3(static_cast<unsigned>(cus)), dim3(kExcessThreads), 0, p.stream,
                       static_cast<const T *>(p.target), static_cast<const T *>(p.draft), p.K, p.L, p.V, p.c,
                       reinterpret_cast<const RowStat *>(p.ws + p.lay.stats),
                       reinterpret_cast<const int32_t *>(p.ws + p.lay.later), static_cast<int>(grid),
                       later_list_entries(nchains, grid, p.L), reinterpret_cast<double *>(p.ws + p.lay.excess_part));
    return hipGetLastError();
}

template <typename T>
hipError_t launch_typed(const Problem &p)
{
    if (p.pend_levels > 0)              // pending modifications: two variants only
        return p.K == 8 ? launch_kp<T, 8, true>(p) : launch_kp<T, 0, true>(p);
    switch (p.K) {                      // the power t^K unrolled for the common draft counts
    case 1: return launch_kp<T, 1, false>(p);
    case 2: return launch_kp<T, 2, false>(p);
    case 3: return launch_kp<T, 3, false>(p);
    case 4: return launch_kp<T, 4, false>(p);
    case 8: return launch_kp<T, 8, false>(p);
    case 16: return launch_kp<T, 16, false>(p);
    default: return launch_kp<T, 0, false>(p);
    }
}

}  // namespace

// Parts k_chain_excess leaves the cancellation-free sum of a marked row in.
int chain_excess_parts(const Problem &) { return kPendParts; }

bool chain_supported(const Problem &p)
{
    const int pv = p.dtype == 1 ? 8 : 4;
    return p.V % pv == 0 && (p.V / pv) >= 7 * kChainThreads &&
           reinterpret_cast<uintptr_t>(p.target) % 16 == 0 && reinterpret_cast<uintptr_t>(p.draft) % 16 == 0;
}

// With pending modifications the whole row pair must be on chip (the extra sweeps read the on-chip copy only).
bool chain_supports_pending(const Problem &p)
{
    if (!chain_supported(p)) return false;
    const int nvec = p.V / (p.dtype == 1 ? 8 : 4);
    const int full_slots = nvec / kChainThreads, nslots = (nvec + kChainThreads - 1) / kChainThreads;
    const int RS = full_slots >= 23 ? 23 : (full_slots >= 15 ? 15 : 7);
    return nslots <= RS + kLdsSlots;
}

// The chain schedule takes about the same time for any number of chains up to one per compute unit
// (each workgroup streams its own rows), the two-pass schedule takes time in proportion to the
// bytes: measured at V = 128256, bf16, L = 8 on 256 compute units they cross at about 170 chains.
bool chain_preferred(const Problem &p)
{
    return chain_supported(p) && static_cast<long long>(p.batch) * p.K * 100 >= static_cast<long long>(resident_workgroups()) * 66;
}

hipError_t launch_chain_main(const Problem &p)
{
    return p.dtype == 1 ? launch_typed<uint16_t>(p) : launch_typed<float>(p);
}

hipError_t launch_chain_excess(const Problem &p)
{
    if (p.pend_levels > 0 || p.batch == 0) return hipSuccess;     // (rows under pending modifications keep the plain sum)
    return p.dtype == 1 ? launch_excess_typed<uint16_t>(p) : launch_excess_typed<float>(p);
}

}  // namespace specgbv
