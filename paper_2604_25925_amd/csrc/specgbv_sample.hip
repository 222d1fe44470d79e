// Draft-side sampling (the drafting step of Algorithm 3): one token per row from
// softmax(logits[row, :] / T) by inverse CDF in token-id order.
//
// One 512-thread workgroup streams one row.  The row is cut into 512-entry segments (one wave x
// 8 entries per lane, so lane order is token order); wave w takes segments w, w + 8, ...; each
// segment's weight sum goes to LDS together with its own integral reference exponent, so no
// row-wide maximum is needed before the pass.  Then the workgroup brings the sums to a common
// scale, finds the segment in which the running sum first exceeds u * total by a scan, and its
// first wave re-reads that one segment and finds the entry.  The row is read once (plus one
// segment); nothing is exchanged between workgroups.
#include "specgbv_internal.hpp"

namespace specgbv {
namespace {

constexpr int kSampThreads = 512;
constexpr int kSampWaves = kSampThreads / kWave;
constexpr int kSampMaxSeg = 2048;            // V <= 2048 * 512 entries per row

// the 8 logits [e0, e0 + 8) of a row; entries at or beyond V read as -inf
template <typename T, bool VEC>
__device__ __forceinline__ void samp_load8(const T *row, long long e0, int V, float (&z)[8])
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

// largest of the logits packed in one 16-byte vector
template <typename T>
__device__ __forceinline__ float vec_max_elem(const U4 &v)
{
    constexpr int PV = Elem<T>::kPerVec;
    float t[PV];
    Elem<T>::unpack(v, t);
    float m = t[0];
#pragma unroll
    for (int j = 1; j < PV; ++j) m = fmaxf(m, t[j]);
    return m;
}

// weights of a lane's 8 entries relative to 2^m2; m2 = NaN asks for the segment's own reference
__device__ __forceinline__ float samp_weigh(const float (&z)[8], float c, float m2_in, float (&w)[8])
{
    float m2 = m2_in;
    if (!(m2 == m2)) {
        float m = -3.0e38f;
#pragma unroll
        for (int j = 0; j < 8; ++j) m = fmaxf(m, z[j]);
        m2 = integral_reference(wave_max(m), c);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = exp2_fast(fmaf(z[j], c, -m2));
    return m2;
}

template <typename T, bool VEC>
__global__ void __launch_bounds__(kSampThreads)
k_sample_rows(const T *__restrict__ logits, int V, float c, int nseg, uint64_t seed, uint64_t offset, uint32_t slot,
              int32_t *__restrict__ out_tokens, double *__restrict__ u_out, double *__restrict__ margin_out)
{
    __shared__ double sh_sum[kSampMaxSeg];
    __shared__ float sh_m2[kSampMaxSeg];
    __shared__ double sh_d[kSampWaves];
    __shared__ double sh_scan[kSampWaves];
    __shared__ float sh_f[kSampWaves];
    __shared__ int sh_seg, sh_first[kSampWaves], sh_last[kSampWaves];
    __shared__ double sh_local_target, sh_total;
    const int row_id = blockIdx.x, tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wid = tid / kWave;
    const T *row = logits + static_cast<long long>(row_id) * V;

    // ---- pass over the row.  Aligned rows: a lane's 8 entries of a segment are kept as loaded (16-byte vectors), 16
    // segments of this wave in flight at a time (8 for float32 rows): a workgroup streams its row alone on its compute
    // unit, so the loads in flight are what hides the memory latency.  Other rows: four segments, entry by entry.
    constexpr int PV = Elem<T>::kPerVec;
    constexpr int NV = 8 / PV;                              // vectors per lane and segment
    constexpr int UN = VEC ? 16 / NV : 4;
    // m2 = NaN: the segment takes its own reference exponent; else the one given (shared by a batch of segments)
    auto reduce_segment = [&](int s, const float (&z)[8], float m2_in) {
        float w[8];
        const float m2 = samp_weigh(z, c, m2_in, w);
        // 512 weights of at most 2^1 each: float32 sums (8 per lane, then over the wave) are good to a few 1e-7 of
        // the segment, far inside the 1e-6 of the total below which a draw counts as undecided
        const float a = wave_sum_f32(((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7])));
        if (lane == 0) { sh_sum[s] = static_cast<double>(a); sh_m2[s] = m2; }
    };
    for (int s0 = wid; s0 < nseg; s0 += UN * kSampWaves) {
        if constexpr (VEC) {
            // V is a multiple of the vector length, so a vector lies wholly inside the row or wholly beyond it
            const uint32_t ninf = PV == 8 ? 0xFF80FF80u : 0xFF800000u;
            U4 raw[UN][NV];
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int s = s0 + i * kSampWaves;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const long long e = static_cast<long long>(s) * kSegElems + lane * 8 + v * PV;
                    raw[i][v] = (s < nseg && e < V) ? load16(row + e) : U4{ninf, ninf, ninf, ninf};
                }
            }
            // one reference exponent for the whole batch (its largest logit): a wave-wide maximum per batch instead
            // of one per segment.  Entries 2^-126 below it round to weight 0, which they are against the total anyway.
            float mb = -3.0e38f;
#pragma unroll
            for (int i = 0; i < UN; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v) mb = fmaxf(mb, vec_max_elem<T>(raw[i][v]));
            const float m2_batch = integral_reference(wave_max(mb), c);
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int s = s0 + i * kSampWaves;
                if (s < nseg) {                               // wave-uniform
                    float z[8];
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        float t[PV];
                        Elem<T>::unpack(raw[i][v], t);
#pragma unroll
                        for (int j = 0; j < PV; ++j) z[v * PV + j] = t[j];
                    }
                    reduce_segment(s, z, m2_batch);
                }
            }
        } else {
            float z[UN][8];
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int s = s0 + i * kSampWaves;
                if (s < nseg) samp_load8<T, VEC>(row, static_cast<long long>(s) * kSegElems + lane * 8, V, z[i]);
            }
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int s = s0 + i * kSampWaves;
                if (s < nseg) reduce_segment(s, z[i], __builtin_nanf(""));   // wave-uniform
            }
        }
    }
    __syncthreads();

    // ---- common scale, total, and the thread whose contiguous segments contain the goal
    const int chunk = (nseg + kSampThreads - 1) / kSampThreads;
    const int s0 = tid * chunk, s1 = min(nseg, s0 + chunk);
    float mloc = -3.0e38f;
    for (int s = s0; s < s1; ++s) mloc = fmaxf(mloc, sh_m2[s]);
    const float M = block_max(mloc, sh_f);
    double mine_seg = 0.0;
    for (int s = s0; s < s1; ++s) mine_seg += ldexp(sh_sum[s], reference_shift(sh_m2[s], M));
    const double W = block_sum(mine_seg, sh_d);
    const double u = philox_uniform(seed, offset, static_cast<uint32_t>(row_id), slot);
    const double goal = u * W;
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
        sh_first[wid] = over ? wid * kWave + __ffsll(static_cast<long long>(over)) - 1 : kSampThreads;
        sh_last[wid] = has ? wid * kWave + 63 - __clzll(static_cast<long long>(has)) : -1;
    }
    __syncthreads();
    int win_t = kSampThreads, last_t = -1;
#pragma unroll
    for (int wv = 0; wv < kSampWaves; ++wv) { win_t = min(win_t, sh_first[wv]); last_t = max(last_t, sh_last[wv]); }
    if (win_t == kSampThreads) win_t = last_t < 0 ? 0 : last_t;     // rounding pushed the goal past the end
    if (tid == win_t) {
        double cum = excl_t, cum_before = excl_t, cum_before_last = excl_t;
        int found = -1, last_pos = s0 < nseg ? s0 : 0;
        for (int s = s0; s < s1; ++s) {
            const double v = ldexp(sh_sum[s], reference_shift(sh_m2[s], M));
            if (v > 0.0) { last_pos = s; cum_before_last = cum; }
            if (cum + v > goal) { found = s; cum_before = cum; break; }
            cum += v;
        }
        if (found < 0) { found = last_pos; cum_before = cum_before_last; }
        const int up = -reference_shift(sh_m2[found], M);
        sh_seg = found;
        sh_local_target = ldexp(goal - cum_before, up);        // goal in the segment's own scale
        sh_total = ldexp(W, up);
    }
    __syncthreads();
    if (wid != 0) return;

    // ---- inside the segment: one wave, lane order = token-id order
    const int seg = sh_seg;
    const double local_target = sh_local_target;
    float z[8], w[8];
    samp_load8<T, VEC>(row, static_cast<long long>(seg) * kSegElems + lane * 8, V, z);
    samp_weigh(z, c, sh_m2[seg], w);
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < 8; ++j) mine += static_cast<double>(w[j]);
    const double incl = wave_inclusive_sum(mine);
    const double excl = incl - mine;
    const unsigned long long cross = __ballot(mine > 0.0 && incl > local_target);
    const unsigned long long pos = __ballot(mine > 0.0);
    int winner;
    if (cross) winner = __ffsll(static_cast<long long>(cross)) - 1;
    else if (pos) winner = 63 - __clzll(static_cast<long long>(pos));
    else winner = 0;
    if (lane == winner) {
        double run = excl, mg = 0.0;
        int y = -1, last = -1;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double prev = run;
            run += static_cast<double>(w[j]);
            if (w[j] > 0.0f) last = j;
            if (y < 0 && run > local_target) {
                y = j;
                const double lo = local_target - prev, hi = run - local_target;
                mg = (lo < hi ? lo : hi) / sh_total;
            }
        }
        if (y < 0) { y = last < 0 ? 0 : last; mg = 0.0; }
        long long tokid = static_cast<long long>(seg) * kSegElems + lane * 8 + y;
        if (tokid >= V) tokid = V - 1;
        out_tokens[row_id] = static_cast<int32_t>(tokid);
        u_out[row_id] = u;
        margin_out[row_id] = mg;
    }
}

template <typename T>
hipError_t launch_sample_typed(const void *logits, int rows, int V, float c, uint64_t seed, uint64_t offset,
                               uint32_t slot, int32_t *out_tokens, double *u_out, double *margin_out, hipStream_t stream)
{
    const bool vec = (V % Elem<T>::kPerVec) == 0 && reinterpret_cast<uintptr_t>(logits) % 16 == 0;
    const int nseg = (V + kSegElems - 1) / kSegElems;
    if (vec)
        hipLaunchKernelGGL((k_sample_rows<T, true>), dim3(rows), dim3(kSampThreads), 0, stream, static_cast<const T *>(logits),
                           V, c, nseg, seed, offset, slot, out_tokens, u_out, margin_out);
    else
        hipLaunchKernelGGL((k_sample_rows<T, false>), dim3(rows), dim3(kSampThreads), 0, stream, static_cast<const T *>(logits),
                           V, c, nseg, seed, offset, slot, out_tokens, u_out, margin_out);
    return hipGetLastError();
}

}  // namespace

int sample_max_vocab() { return kSampMaxSeg * kSegElems; }

hipError_t launch_sample_rows(const void *logits, int rows, int V, int dtype, float c, uint64_t seed, uint64_t offset,
                              uint32_t slot, int32_t *out_tokens, double *u_out, double *margin_out, hipStream_t stream)
{
    return dtype == 1 ? launch_sample_typed<uint16_t>(logits, rows, V, c, seed, offset, slot, out_tokens, u_out, margin_out, stream)
                      : launch_sample_typed<float>(logits, rows, V, c, seed, offset, slot, out_tokens, u_out, margin_out, stream);
}

}  // namespace specgbv
