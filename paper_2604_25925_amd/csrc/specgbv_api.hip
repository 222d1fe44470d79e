// C ABI of libspecgbv.so: argument checks, workspace layout, kernel sequencing.
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "../../include/specgbv.h"
#include "specgbv_internal.hpp"

namespace specgbv {

static thread_local char g_err[512] = "";

static specgbv_status fail(specgbv_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

static size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// Scratch memory of specgbv_verify_static: the verification workspace for callers that cannot allocate one.
// One copy per GPU the library runs on, held until the process ends; every call on a GPU shares that GPU's copy.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char g_static_scratch[SPECGBV_STATIC_SCRATCH_BYTES];
static std::atomic<void *> g_static_scratch_ptr[kMaxDevices];     // device address per GPU, looked up on first use

Workspace make_workspace(int batch, int K, int L, int V)
{
    Workspace w{};
    const size_t n = static_cast<size_t>(batch) * K * L;
    size_t off = 0;
    auto take = [&off](size_t bytes) { const size_t o = off; off = align256(off + bytes); return o; };
    w.nseg = (V + kSegElems - 1) / kSegElems;
    w.stats = take(n * sizeof(RowStat));
    w.s = take(n * sizeof(double));
    w.excess = take(n * sizeof(double));
    w.excess_part = take(n * kPendParts * sizeof(double));
    w.log_nu = take(n * sizeof(double));
    w.log_P = take(n * sizeof(double));
    w.h = take(n * sizeof(double));
    w.eta = take(n * sizeof(double));
    w.state = take(n * sizeof(int32_t));
    w.sel = take(static_cast<size_t>(batch) * sizeof(Selection));
    w.partial = take(static_cast<size_t>(batch) * w.nseg * sizeof(SegPartial));
    w.res_norm = take(static_cast<size_t>(batch) * sizeof(double));
    w.u_final = take(static_cast<size_t>(batch) * sizeof(double));
    w.margin = take(static_cast<size_t>(batch) * sizeof(double));
    w.fallback = take(static_cast<size_t>(batch) * sizeof(int32_t));
    w.carry = take(static_cast<size_t>(batch) * sizeof(double));
    w.mcount = take(static_cast<size_t>(batch) * sizeof(int32_t));
    w.counter = take(static_cast<size_t>(batch) * sizeof(int32_t));
    w.pend = take(n * kMaxPend * sizeof(PendRow));
    w.pend_off = take(static_cast<size_t>(kMaxPend) * (static_cast<size_t>(batch) + 1) * sizeof(int32_t));
    w.pend_part = take(n * kPendParts * sizeof(double));
    w.pend_cnt = take(n * sizeof(int32_t));
    w.stat_part = take(n * 2 * kRowParts * sizeof(Row0Part));
    w.row0 = take(static_cast<size_t>(batch) * 2 * kRow0Parts * sizeof(Row0Part));
    // (lists of g <= kMaxChainGrid workgroups, each 1 + ceil(chains / g) (L - 1) entries: at most this many in all)
    w.later = take((static_cast<size_t>(kMaxChainGrid) +
                    (static_cast<size_t>(batch) * K + kMaxChainGrid) * static_cast<size_t>(L > 1 ? L - 1 : 0)) * sizeof(int32_t));
    w.kseq_pos = take(static_cast<size_t>(batch) * L * 2 * sizeof(int32_t));
    w.total = off;
    return w;
}

static bool shape_ok(int batch, int K, int L, int V)
{
    return batch >= 0 && K >= 1 && L >= 1 && V >= 1;
}

static specgbv_status check_limits(int batch, int K, int L, int V)
{
    if (K > SPECGBV_MAX_K) return fail(SPECGBV_EUNSUPPORTED, "K=%d exceeds SPECGBV_MAX_K=%d", K, SPECGBV_MAX_K);
    if (L > SPECGBV_MAX_L) return fail(SPECGBV_EUNSUPPORTED, "L=%d exceeds SPECGBV_MAX_L=%d", L, SPECGBV_MAX_L);
    if (K * L > 1024) return fail(SPECGBV_EUNSUPPORTED, "K*L=%d exceeds 1024", K * L);
    const double rows = static_cast<double>(batch) * K * (L + 1);
    if (rows > 2.0e9 || static_cast<double>(batch) > 65535.0)
        return fail(SPECGBV_EUNSUPPORTED, "batch=%d is too large for one launch", batch);
    if (rows * V > 9.0e18) return fail(SPECGBV_EUNSUPPORTED, "tensor too large");
    return SPECGBV_OK;
}

}  // namespace specgbv

using namespace specgbv;

extern "C" {

size_t specgbv_workspace_bytes(int batch, int K, int L, int V, specgbv_dtype dtype)
{
    if (!shape_ok(batch, K, L, V) || (dtype != SPECGBV_F32 && dtype != SPECGBV_BF16)) return 0;
    if (check_limits(batch, K, L, V) != SPECGBV_OK) return 0;
    return make_workspace(batch < 1 ? 1 : batch, K, L, V).total;
}

size_t specgbv_pending_state_bytes(int batch)
{
    if (batch < 0) return 0;
    const size_t b = static_cast<size_t>(batch < 1 ? 1 : batch);
    return align256(b * kMaxPend * (sizeof(double) + sizeof(int32_t)));
}

specgbv_status specgbv_verify_ex(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream,
    const specgbv_options *options)
{
    if (!shape_ok(batch, K, L, V))
        return fail(SPECGBV_EINVAL, "sizes must satisfy batch >= 0, K, L, V >= 1 (got batch=%d K=%d L=%d V=%d)",
                    batch, K, L, V);
    if (dtype != SPECGBV_F32 && dtype != SPECGBV_BF16) return fail(SPECGBV_EINVAL, "unknown dtype %d", (int)dtype);
    if (!(temperature > 0.0f) || !std::isfinite(temperature))
        return fail(SPECGBV_EINVAL, "temperature must be finite and > 0 (got %g)", (double)temperature);
    const int algo = options ? options->algo : SPECGBV_ALGO_AUTO;
    if (algo < SPECGBV_ALGO_AUTO || algo > SPECGBV_ALGO_CHAIN) return fail(SPECGBV_EINVAL, "unknown algo %d", algo);
    specgbv_status st = check_limits(batch, K, L, V);
    if (st != SPECGBV_OK) return st;
    if (batch == 0) return SPECGBV_OK;
    if (!target_logits || !draft_logits || !draft_tokens || !accepted_len || !accepted_draft_idx || !out_tokens)
        return fail(SPECGBV_EINVAL, "null input or output pointer");
    const size_t esz = dtype == SPECGBV_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(target_logits) % esz || reinterpret_cast<uintptr_t>(draft_logits) % esz ||
        reinterpret_cast<uintptr_t>(draft_tokens) % 4 || reinterpret_cast<uintptr_t>(accepted_len) % 4 ||
        reinterpret_cast<uintptr_t>(accepted_draft_idx) % 4 || reinterpret_cast<uintptr_t>(out_tokens) % 4)
        return fail(SPECGBV_EINVAL, "pointer not aligned to its element size");

    Problem p{};
    p.lay = make_workspace(batch, K, L, V);
    if (!workspace) return fail(SPECGBV_EWORKSPACE, "workspace is null (need %zu bytes)", p.lay.total);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(SPECGBV_EWORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < p.lay.total)
        return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, p.lay.total);
    p.target = target_logits; p.draft = draft_logits; p.tokens = draft_tokens;
    p.K = K; p.L = L; p.V = V; p.batch = batch; p.dtype = dtype == SPECGBV_BF16 ? 1 : 0;
    const double c_exact = 1.4426950408889634074 / static_cast<double>(temperature);
    p.c = static_cast<float>(c_exact);
    p.c_rel = c_exact / static_cast<double>(p.c) - 1.0;
    p.seed = rng_seed; p.offset = rng_offset;
    p.accepted_len = accepted_len; p.accepted_draft_idx = accepted_draft_idx; p.out_tokens = out_tokens;
    p.ws = static_cast<char *>(workspace);
    p.stream = static_cast<hipStream_t>(hip_stream);

    static_assert(SPECGBV_MAX_PENDING == kMaxPend, "header and kernels disagree on the number of pending levels");
    static_assert(SPECGBV_MAX_K == kMaxDrafts, "header and kernels disagree on the number of drafts");
    p.pend_carry = options ? options->pending_carry_log_nu : nullptr;
    p.pend_count = options ? options->pending_count : nullptr;
    p.pend_levels = 0;
    p.state_carry = nullptr; p.state_count = nullptr;
    if ((p.pend_carry == nullptr) != (p.pend_count == nullptr))
        return fail(SPECGBV_EINVAL, "pending_carry_log_nu and pending_count must be given together");
    if (p.pend_carry) {
        if (options->pending_state) return fail(SPECGBV_EINVAL, "give pending_state or the pending arrays, not both");
        if (reinterpret_cast<uintptr_t>(p.pend_carry) % 8 || reinterpret_cast<uintptr_t>(p.pend_count) % 4)
            return fail(SPECGBV_EINVAL, "pointer not aligned to its element size");
        if (options->pending_levels < 0 || options->pending_levels > SPECGBV_MAX_PENDING)
            return fail(SPECGBV_EUNSUPPORTED, "pending_levels=%d exceeds SPECGBV_MAX_PENDING=%d", options->pending_levels,
                        SPECGBV_MAX_PENDING);
        p.pend_levels = options->pending_levels > 0 ? options->pending_levels : 1;
    } else if (options && options->pending_levels != 0) {
        return fail(SPECGBV_EINVAL, "pending_levels given without the pending arrays");
    } else if (options && options->pending_state) {
        if (reinterpret_cast<uintptr_t>(options->pending_state) % 8)
            return fail(SPECGBV_EINVAL, "pending_state must be 8-byte aligned");
        if (L - 1 > SPECGBV_MAX_PENDING)
            return fail(SPECGBV_EUNSUPPORTED, "pending_state needs L - 1 <= SPECGBV_MAX_PENDING=%d (L=%d)", SPECGBV_MAX_PENDING, L);
        p.state_carry = static_cast<double *>(options->pending_state);
        p.state_count = reinterpret_cast<int32_t *>(p.state_carry + static_cast<size_t>(kMaxPend) * batch);
        p.pend_carry = p.state_carry; p.pend_count = p.state_count;
        p.pend_levels = L - 1;               // at most L - 1 modifications are alive at once; 0 for L = 1
    }
    const bool pending = p.pend_levels > 0;
    p.shared_row0 = options && options->shared_row0 != 0 && !pending;
    bool use_chain = false;
    if (algo == SPECGBV_ALGO_CHAIN) {
        if (!(pending ? chain_supports_pending(p) : chain_supported(p)))
            return fail(SPECGBV_EUNSUPPORTED, pending ? "the chain schedule with pending modifications needs the whole row pair on chip"
                                                      : "the chain schedule does not support this shape");
        use_chain = true;
    } else if (algo == SPECGBV_ALGO_AUTO) {
        // With pending modifications the two-pass schedule is the default: its extra passes spread over the whole
        // chip, while a chain pays for its modified rows alone (measured: the chain is ahead only while at most
        // about three rows per draft are modified, and a batch waits for its most modified prefix).
        use_chain = !pending && chain_preferred(p);
    }

    p.s_parts = use_chain ? 1 : split_sum_parts(p);
    p.e_parts = (use_chain && !pending) ? chain_excess_parts(p) : 0;
    p.e_coop = use_chain ? 0 : 1;

    hipError_t e;
    if (options && options->ev_main_start) {
        e = hipEventRecord(static_cast<hipEvent_t>(options->ev_main_start), p.stream);
        if (e != hipSuccess) return fail(SPECGBV_EHIP, "hipEventRecord: %s", hipGetErrorString(e));
    }
    e = use_chain ? launch_chain_main(p) : launch_split_main(p);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "main kernel launch: %s", hipGetErrorString(e));
    if (options && options->ev_main_stop) {
        e = hipEventRecord(static_cast<hipEvent_t>(options->ev_main_stop), p.stream);
        if (e != hipSuccess) return fail(SPECGBV_EHIP, "hipEventRecord: %s", hipGetErrorString(e));
    }
    if (use_chain) {
        e = launch_chain_excess(p);
        if (e != hipSuccess) return fail(SPECGBV_EHIP, "follow-up kernel launch: %s", hipGetErrorString(e));
    }
    e = launch_decide_and_sample(p);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "decision/sampling kernel launch: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

specgbv_status specgbv_verify_kseq(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset, int ndrafts,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!shape_ok(batch, K, L, V))
        return fail(SPECGBV_EINVAL, "sizes must satisfy batch >= 0, K, L, V >= 1 (got batch=%d K=%d L=%d V=%d)",
                    batch, K, L, V);
    if (ndrafts < 1 || ndrafts > K) return fail(SPECGBV_EINVAL, "ndrafts must lie in [1, K] (got %d, K=%d)", ndrafts, K);
    if (dtype != SPECGBV_F32 && dtype != SPECGBV_BF16) return fail(SPECGBV_EINVAL, "unknown dtype %d", (int)dtype);
    if (!(temperature > 0.0f) || !std::isfinite(temperature))
        return fail(SPECGBV_EINVAL, "temperature must be finite and > 0 (got %g)", (double)temperature);
    specgbv_status st = check_limits(batch, K, L, V);
    if (st != SPECGBV_OK) return st;
    if (batch == 0) return SPECGBV_OK;
    if (!target_logits || !draft_logits || !draft_tokens || !accepted_len || !accepted_draft_idx || !out_tokens)
        return fail(SPECGBV_EINVAL, "null input or output pointer");
    const size_t esz = dtype == SPECGBV_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(target_logits) % esz || reinterpret_cast<uintptr_t>(draft_logits) % esz ||
        reinterpret_cast<uintptr_t>(draft_tokens) % 4 || reinterpret_cast<uintptr_t>(accepted_len) % 4 ||
        reinterpret_cast<uintptr_t>(accepted_draft_idx) % 4 || reinterpret_cast<uintptr_t>(out_tokens) % 4)
        return fail(SPECGBV_EINVAL, "pointer not aligned to its element size");
    Problem p{};
    p.lay = make_workspace(batch, K, L, V);
    if (!workspace) return fail(SPECGBV_EWORKSPACE, "workspace is null (need %zu bytes)", p.lay.total);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(SPECGBV_EWORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < p.lay.total)
        return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, p.lay.total);
    p.target = target_logits; p.draft = draft_logits; p.tokens = draft_tokens;
    p.K = K; p.L = L; p.V = V; p.batch = batch; p.dtype = dtype == SPECGBV_BF16 ? 1 : 0;
    const double c_exact = 1.4426950408889634074 / static_cast<double>(temperature);
    p.c = static_cast<float>(c_exact);
    p.c_rel = c_exact / static_cast<double>(p.c) - 1.0;
    p.seed = rng_seed; p.offset = rng_offset;
    p.accepted_len = accepted_len; p.accepted_draft_idx = accepted_draft_idx; p.out_tokens = out_tokens;
    p.ws = static_cast<char *>(workspace);
    p.stream = static_cast<hipStream_t>(hip_stream);
    p.s_parts = 1;
    p.kseq_ndrafts = ndrafts;
    hipError_t e = launch_kseq_rows(p, ndrafts);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "root-finding kernel launch: %s", hipGetErrorString(e));
    e = launch_decide_and_sample(p);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "decision/sampling kernel launch: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

specgbv_status specgbv_read_kseq_intermediates(
    const void *workspace, size_t workspace_bytes, int batch, int K, int L, int V,
    const specgbv_kseq_intermediates *out, void *hip_stream)
{
    if (!shape_ok(batch, K, L, V) || batch < 1) return fail(SPECGBV_EINVAL, "bad shape");
    if (!workspace || !out) return fail(SPECGBV_EINVAL, "null pointer");
    const Workspace lay = make_workspace(batch, K, L, V);
    if (workspace_bytes < lay.total) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, lay.total);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const char *ws = static_cast<const char *>(workspace);
    const size_t n = static_cast<size_t>(batch) * K * L, m = static_cast<size_t>(batch) * L;
    hipError_t e = hipSuccess;
    auto copy = [&](void *dst, size_t off, size_t bytes) {
        if (dst && e == hipSuccess) e = hipMemcpyAsync(dst, ws + off, bytes, hipMemcpyDeviceToHost, stream);
    };
    copy(out->rho_all, lay.s, n * sizeof(double));
    copy(out->beta_all, lay.excess, n * sizeof(double));
    copy(out->accept, lay.h, n * sizeof(double));
    copy(out->eta, lay.eta, n * sizeof(double));
    copy(out->state, lay.state, n * sizeof(int32_t));
    copy(out->retained, lay.kseq_pos, m * sizeof(int32_t));
    copy(out->lead, lay.kseq_pos + m * sizeof(int32_t), m * sizeof(int32_t));
    copy(out->res_norm, lay.res_norm, batch * sizeof(double));
    copy(out->u_final, lay.u_final, batch * sizeof(double));
    copy(out->margin, lay.margin, batch * sizeof(double));
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "reading intermediates: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

specgbv_status specgbv_verify(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return specgbv_verify_ex(target_logits, draft_logits, draft_tokens, K, L, V, batch, dtype, temperature,
                             rng_seed, rng_offset, accepted_len, accepted_draft_idx, out_tokens, workspace,
                             workspace_bytes, hip_stream, nullptr);
}

specgbv_status specgbv_read_intermediates(
    const void *workspace, size_t workspace_bytes, int batch, int K, int L, int V,
    specgbv_dtype dtype, const specgbv_intermediates *out, void *hip_stream)
{
    (void)dtype;
    if (!shape_ok(batch, K, L, V) || batch < 1) return fail(SPECGBV_EINVAL, "bad shape");
    if (!workspace || !out) return fail(SPECGBV_EINVAL, "null pointer");
    const Workspace lay = make_workspace(batch, K, L, V);
    if (workspace_bytes < lay.total) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, lay.total);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const char *ws = static_cast<const char *>(workspace);
    const size_t n = static_cast<size_t>(batch) * K * L;
    hipError_t e = hipSuccess;
    auto copy = [&](void *dst, size_t off, size_t bytes) {
        if (dst && e == hipSuccess) e = hipMemcpyAsync(dst, ws + off, bytes, hipMemcpyDeviceToHost, stream);
    };
    // statistics are stored interleaved in base 2; unpack on the host
    RowStat *tmp = nullptr;
    if (out->lse_q || out->lse_p) {
        tmp = static_cast<RowStat *>(malloc(n * sizeof(RowStat)));
        if (!tmp) return fail(SPECGBV_EINVAL, "host allocation failed");
        copy(tmp, lay.stats, n * sizeof(RowStat));
    }
    copy(out->log_nu, lay.log_nu, n * sizeof(double));
    copy(out->log_P, lay.log_P, n * sizeof(double));
    copy(out->s, lay.s, n * sizeof(double));
    copy(out->h, lay.h, n * sizeof(double));
    copy(out->eta, lay.eta, n * sizeof(double));
    copy(out->state, lay.state, n * sizeof(int32_t));
    copy(out->res_norm, lay.res_norm, batch * sizeof(double));
    copy(out->u_final, lay.u_final, batch * sizeof(double));
    copy(out->margin, lay.margin, batch * sizeof(double));
    copy(out->fallback, lay.fallback, batch * sizeof(int32_t));
    copy(out->carry_log_nu, lay.carry, batch * sizeof(double));
    copy(out->modify_count, lay.mcount, batch * sizeof(int32_t));
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        free(tmp);
        return fail(SPECGBV_EHIP, "reading intermediates: %s", hipGetErrorString(e));
    }
    if (tmp) {
        const double ln2 = 0.693147180559945309417;
        for (size_t j = 0; j < n; ++j) {
            if (out->lse_q) out->lse_q[j] = tmp[j].lse2_q * ln2;
            if (out->lse_p) out->lse_p[j] = tmp[j].lse2_p * ln2;
        }
        free(tmp);
    }
    if (out->s) {
        const double nan = std::nan("");
        for (size_t j = 0; j < n; j += L) out->s[j] = nan;      // row 0 carries no Eq. (hik) sum
    }
    return SPECGBV_OK;
}

specgbv_status specgbv_workspace_carry(void *workspace, size_t workspace_bytes, int batch, int K, int L, int V,
                                       double **carry_log_nu, int32_t **modify_count)
{
    if (!shape_ok(batch, K, L, V) || batch < 1) return fail(SPECGBV_EINVAL, "bad shape");
    if (!workspace || !carry_log_nu || !modify_count) return fail(SPECGBV_EINVAL, "null pointer");
    const Workspace lay = make_workspace(batch, K, L, V);
    if (workspace_bytes < lay.total) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, lay.total);
    *carry_log_nu = reinterpret_cast<double *>(static_cast<char *>(workspace) + lay.carry);
    *modify_count = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + lay.mcount);
    return SPECGBV_OK;
}

static specgbv_status check_modify_shape(int batch, int K, int M, int bonus_row, int V)
{
    if (batch < 0 || K < 1 || M < 1 || V < 1) return fail(SPECGBV_EINVAL, "bad shape batch=%d K=%d M=%d V=%d", batch, K, M, V);
    if (bonus_row != 0 && bonus_row != 1) return fail(SPECGBV_EINVAL, "bonus_row must be 0 or 1 (got %d)", bonus_row);
    if (K > SPECGBV_MAX_K) return fail(SPECGBV_EUNSUPPORTED, "K=%d exceeds SPECGBV_MAX_K=%d", K, SPECGBV_MAX_K);
    if (M > SPECGBV_MAX_L) return fail(SPECGBV_EUNSUPPORTED, "M=%d exceeds SPECGBV_MAX_L=%d", M, SPECGBV_MAX_L);
    const double rows = static_cast<double>(batch) * K * (2 * M + 1);
    if (rows > 2.0e9 || rows * V > 9.0e18) return fail(SPECGBV_EUNSUPPORTED, "tensor too large");
    return SPECGBV_OK;
}

size_t specgbv_modify_workspace_bytes(int batch, int K, int M, int bonus_row)
{
    if (check_modify_shape(batch, K, M, bonus_row, 1) != SPECGBV_OK) return 0;
    return modify_workspace_bytes(batch < 1 ? 1 : batch, K, M, bonus_row);
}

specgbv_status specgbv_modify_target(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int M, int bonus_row, int V, int batch, specgbv_dtype dtype, float temperature,
    const double *carry_log_nu, const int32_t *modify_count,
    float *out_logq, float *out_logp, double *norm_out, int32_t *fallback_out,
    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const specgbv_status st = check_modify_shape(batch, K, M, bonus_row, V);
    if (st != SPECGBV_OK) return st;
    if (dtype != SPECGBV_F32 && dtype != SPECGBV_BF16) return fail(SPECGBV_EINVAL, "unknown dtype %d", static_cast<int>(dtype));
    if (!(temperature > 0.0f) || !std::isfinite(temperature)) return fail(SPECGBV_EINVAL, "temperature must be positive and finite");
    if (batch == 0) return SPECGBV_OK;
    if (!target_logits || !draft_logits || !draft_tokens || !carry_log_nu || !modify_count || !out_logq)
        return fail(SPECGBV_EINVAL, "null pointer");
    const size_t esz = dtype == SPECGBV_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(target_logits) % esz || reinterpret_cast<uintptr_t>(draft_logits) % esz ||
        reinterpret_cast<uintptr_t>(out_logq) % 4 || reinterpret_cast<uintptr_t>(out_logp) % 4 ||
        reinterpret_cast<uintptr_t>(carry_log_nu) % 8 || reinterpret_cast<uintptr_t>(modify_count) % 4 ||
        reinterpret_cast<uintptr_t>(norm_out) % 8 || reinterpret_cast<uintptr_t>(fallback_out) % 4)
        return fail(SPECGBV_EINVAL, "pointer not aligned to its element size");
    const size_t need = modify_workspace_bytes(batch, K, M, bonus_row);
    if (!workspace) return fail(SPECGBV_EWORKSPACE, "workspace is null (need %zu bytes)", need);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(SPECGBV_EWORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < need) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, need);
    const float c = static_cast<float>(1.44269504088896340736 / static_cast<double>(temperature));
    const hipError_t e = launch_modify(target_logits, draft_logits, draft_tokens, K, M, bonus_row, V, batch,
                                       dtype == SPECGBV_BF16 ? 1 : 0, c, carry_log_nu, modify_count, out_logq, out_logp,
                                       norm_out, fallback_out, static_cast<char *>(workspace),
                                       static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "modification kernel launch: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

size_t specgbv_carry_workspace_bytes(int batch, int M)
{
    if (batch < 0 || M < 1 || M > SPECGBV_MAX_L) return 0;
    return align256(static_cast<size_t>(batch < 1 ? 1 : batch) * M * sizeof(double));
}

specgbv_status specgbv_carry_advance(
    const void *rows_q, const void *rows_p, const int32_t *draft_tokens,
    const int32_t *accepted_len, const int32_t *accepted_draft_idx, const int32_t *out_tokens,
    int K, int M, int bonus_row, int V, int batch, specgbv_dtype dtype, float temperature,
    double *carry_log_nu, int32_t *modify_count, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const specgbv_status st = check_modify_shape(batch, K, M, bonus_row, V);
    if (st != SPECGBV_OK) return st;
    if (dtype != SPECGBV_F32 && dtype != SPECGBV_BF16) return fail(SPECGBV_EINVAL, "unknown dtype %d", static_cast<int>(dtype));
    if (!(temperature > 0.0f) || !std::isfinite(temperature)) return fail(SPECGBV_EINVAL, "temperature must be positive and finite");
    if (batch > 65535) return fail(SPECGBV_EUNSUPPORTED, "batch=%d is too large for one launch", batch);
    if (batch == 0) return SPECGBV_OK;
    if (!rows_q || !rows_p || !draft_tokens || !accepted_len || !accepted_draft_idx || !out_tokens || !carry_log_nu || !modify_count)
        return fail(SPECGBV_EINVAL, "null pointer");
    const size_t esz = dtype == SPECGBV_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(rows_q) % esz || reinterpret_cast<uintptr_t>(rows_p) % esz ||
        reinterpret_cast<uintptr_t>(carry_log_nu) % 8 || reinterpret_cast<uintptr_t>(modify_count) % 4)
        return fail(SPECGBV_EINVAL, "pointer not aligned to its element size");
    const size_t need = specgbv_carry_workspace_bytes(batch, M);
    if (!workspace) return fail(SPECGBV_EWORKSPACE, "workspace is null (need %zu bytes)", need);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(SPECGBV_EWORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < need) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, need);
    const float c = static_cast<float>(1.44269504088896340736 / static_cast<double>(temperature));
    const hipError_t e = launch_carry_advance(rows_q, rows_p, draft_tokens, accepted_len, accepted_draft_idx, out_tokens, K, M,
                                              bonus_row, V, batch, dtype == SPECGBV_BF16 ? 1 : 0, c, carry_log_nu, modify_count,
                                              static_cast<double *>(workspace), static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "carry kernel launch: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

static specgbv_status check_sample_shape(int rows, int V)
{
    if (rows < 0 || V < 1) return fail(SPECGBV_EINVAL, "bad shape rows=%d V=%d", rows, V);
    if (V > sample_max_vocab()) return fail(SPECGBV_EUNSUPPORTED, "V=%d exceeds the sampler's limit of %d", V, sample_max_vocab());
    return SPECGBV_OK;
}

// sampler workspace: uniforms [rows] and margins [rows], float64
static size_t sample_margin_offset(int rows) { return align256(static_cast<size_t>(rows) * sizeof(double)); }

size_t specgbv_sample_workspace_bytes(int rows, int V)
{
    if (check_sample_shape(rows, V) != SPECGBV_OK) return 0;
    return 2 * sample_margin_offset(rows < 1 ? 1 : rows);
}

specgbv_status specgbv_sample_tokens(
    const void *logits, int rows, int V, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset, uint32_t position, int32_t *out_tokens,
    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const specgbv_status st = check_sample_shape(rows, V);
    if (st != SPECGBV_OK) return st;
    if (dtype != SPECGBV_F32 && dtype != SPECGBV_BF16) return fail(SPECGBV_EINVAL, "unknown dtype %d", static_cast<int>(dtype));
    if (!(temperature > 0.0f) || !std::isfinite(temperature)) return fail(SPECGBV_EINVAL, "temperature must be positive and finite");
    if (position >= 0x80000000u) return fail(SPECGBV_EINVAL, "position must be below 2^31");
    if (rows == 0) return SPECGBV_OK;
    if (!logits || !out_tokens) return fail(SPECGBV_EINVAL, "null pointer");
    const size_t esz = dtype == SPECGBV_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits) % esz || reinterpret_cast<uintptr_t>(out_tokens) % 4)
        return fail(SPECGBV_EINVAL, "pointer not aligned to its element size");
    const size_t need = specgbv_sample_workspace_bytes(rows, V);
    if (!workspace) return fail(SPECGBV_EWORKSPACE, "workspace is null (need %zu bytes)", need);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(SPECGBV_EWORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < need) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, need);
    const float c = static_cast<float>(1.44269504088896340736 / static_cast<double>(temperature));
    char *ws = static_cast<char *>(workspace);
    const hipError_t e = launch_sample_rows(logits, rows, V, dtype == SPECGBV_BF16 ? 1 : 0, c, rng_seed, rng_offset,
                                            0x80000000u | position, out_tokens, reinterpret_cast<double *>(ws),
                                            reinterpret_cast<double *>(ws + sample_margin_offset(rows)),
                                            static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "sampling kernel launch: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

specgbv_status specgbv_read_sample_intermediates(const void *workspace, size_t workspace_bytes, int rows, int V,
                                                 double *u_host, double *margin_host, void *hip_stream)
{
    if (check_sample_shape(rows, V) != SPECGBV_OK || rows < 1) return fail(SPECGBV_EINVAL, "bad shape");
    if (!workspace) return fail(SPECGBV_EINVAL, "null pointer");
    const size_t need = specgbv_sample_workspace_bytes(rows, V);
    if (workspace_bytes < need) return fail(SPECGBV_EWORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, need);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const char *ws = static_cast<const char *>(workspace);
    hipError_t e = hipSuccess;
    if (u_host) e = hipMemcpyAsync(u_host, ws, rows * sizeof(double), hipMemcpyDeviceToHost, stream);
    if (margin_host && e == hipSuccess)
        e = hipMemcpyAsync(margin_host, ws + sample_margin_offset(rows), rows * sizeof(double), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "copy of the sampling intermediates: %s", hipGetErrorString(e));
    return SPECGBV_OK;
}

specgbv_status specgbv_verify_static(
    const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
    int K, int L, int V, int batch, specgbv_dtype dtype, float temperature,
    uint64_t rng_seed, uint64_t rng_offset,
    int32_t *accepted_len, int32_t *accepted_draft_idx, int32_t *out_tokens, void *hip_stream)
{
    if (!shape_ok(batch, K, L, V))
        return fail(SPECGBV_EINVAL, "sizes must satisfy batch >= 0, K, L, V >= 1 (got batch=%d K=%d L=%d V=%d)",
                    batch, K, L, V);
    const specgbv_status st = check_limits(batch, K, L, V);
    if (st != SPECGBV_OK) return st;
    const size_t need = make_workspace(batch < 1 ? 1 : batch, K, L, V).total;
    if (need > sizeof g_static_scratch)
        return fail(SPECGBV_EUNSUPPORTED,
                    "this shape needs %zu bytes of scratch memory, the built-in buffer holds SPECGBV_STATIC_SCRATCH_BYTES = %zu: "
                    "use specgbv_verify with a caller-owned workspace",
                    need, sizeof g_static_scratch);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SPECGBV_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(SPECGBV_EUNSUPPORTED, "device index %d is beyond %d", dev, kMaxDevices - 1);
    // Every GPU holds its own copy of the array at its own address: looked up once per device, with that device
    // current; from then on only the looked-up address is used (the array's name is not a device address in host code).
    void *scratch = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!scratch) {
        e = hipGetSymbolAddress(&scratch, HIP_SYMBOL(g_static_scratch));
        if (e != hipSuccess || !scratch)
            return fail(SPECGBV_EHIP, "hipGetSymbolAddress(built-in scratch buffer): %s", hipGetErrorString(e));
        g_static_scratch_ptr[dev].store(scratch, std::memory_order_release);
    }
    return specgbv_verify_ex(target_logits, draft_logits, draft_tokens, K, L, V, batch, dtype, temperature, rng_seed,
                             rng_offset, accepted_len, accepted_draft_idx, out_tokens, scratch, sizeof g_static_scratch,
                             hip_stream, nullptr);
}

const char *specgbv_last_error(void) { return g_err; }

const char *specgbv_version(void) { return "specgbv 0.5 (gfx950)"; }

}  // extern "C"
