// Host-side declarations shared by the translation units of libspecgbv.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "specgbv_device.hpp"

namespace specgbv {

// Device workspace carved into arrays; offsets in bytes, all 256-byte aligned.
struct Workspace {
    size_t stats;      // RowStat [B*K*L]
    size_t s;          // double  [B*K*L]   (position i = row i; position 0 unused)
    size_t excess;     // double  [B*K*L]   nu^2 (s - g) summed without cancellation where the sum kernels took it, else -1
    size_t excess_part;// double  [B*K*L][kPendParts]  the same in parts (small batches)
    size_t log_nu;     // double  [B*K*L]
    size_t log_P;      // double  [B*K*L]
    size_t h;          // double  [B*K*L]
    size_t eta;        // double  [B*K*L]
    size_t state;      // int32   [B*K*L]
    size_t sel;        // Selection [B]
    size_t partial;    // SegPartial [B*nseg]
    size_t res_norm;   // double [B]
    size_t u_final;    // double [B]
    size_t margin;     // double [B]
    size_t fallback;   // int32  [B]
    size_t carry;      // double [B]  ln of q(t^tau, y) / p(t^tau, y) for Algorithm 2 (0 when tau = L)
    size_t mcount;     // int32  [B]  L - tau - 1 rows of the next iteration to modify (0 when tau >= L - 1)
    size_t counter;    // int32  [B]  final-token workgroups that have stored their partial sums; zeroed by the
                       //             streaming kernels of every call
    size_t pend;       // PendRow [kMaxPend][B*K*L]  rows under pending modifications (written only by calls that carry some)
    size_t pend_off;   // int32  [kMaxPend][B+1]  per level: rows the level modifies in the prefixes before b (two-pass schedule)
    size_t pend_part;  // double [B*K*L][kPendParts]  partial normalisers of a modified row shared among workgroups
    size_t pend_cnt;   // int32  [B*K*L]  workgroups of a shared row that have stored their partial normaliser
    size_t stat_part;  // Row0Part [B*K*L][2][kRowParts]  partial row statistics (two-pass schedule, small batches)
    size_t row0;       // Row0Part [B][2][kRow0Parts]  partial statistics of the rows 0 a prefix's drafts share (chain schedule)
    size_t later;      // int32 [workgroups][1 + rows a workgroup sums]  chain schedule: per workgroup, the number of rows
                       //             whose Eq. (hik) sum is taken again without cancellation, then their row indices
    size_t kseq_pos;   // int32 [2][B*L]  comparison verifier: drafts retained at each position, and the lowest of them
    size_t total;
    int nseg;
};

constexpr int kMaxChainGrid = 1024;            // workgroups of the chain kernel at most (one per compute unit)
constexpr int kPendParts = 16;                 // workgroups a modified row's normaliser is shared among, at most
constexpr int kRowParts = 16;                  // workgroups a row is shared among at most when the batch is small
constexpr int kRow0Parts = 16;                 // slices a shared row 0 is reduced in
struct Row0Part { double ref; double Z; };     // sum over the slice of 2^(c z - ref), ref an integer

constexpr int kSegThreads = 256;               // final-token kernels: 4 waves per workgroup
constexpr int kSegElems = kWave * 8;           // vocabulary entries per residual segment (one wave)

Workspace make_workspace(int batch, int K, int L, int V);

struct Problem {
    const void *target;
    const void *draft;
    const int32_t *tokens;
    int K, L, V, batch;
    int dtype;          // 0 = float32, 1 = bfloat16
    float c;            // log2(e) / temperature
    double c_rel;       // (log2(e) / temperature) / c - 1: what the rounding of c to float32 leaves out (token_scaled)
    uint64_t seed, offset;
    int32_t *accepted_len;
    int32_t *accepted_draft_idx;
    int32_t *out_tokens;
    char *ws;
    Workspace lay;
    hipStream_t stream;
    // pending modifications, innermost first: level l changes the first pend_count[l][b] rows of every draft
    int pend_levels;               // 0: none
    const double *pend_carry;      // [pend_levels][batch] ln of the block ratio Algorithm 2 starts from
    const int32_t *pend_count;     // [pend_levels][batch]
    // when not null: the state the call updates in place (kMaxPend levels: carried ratios, then counts)
    double *state_carry;           // [kMaxPend][batch]
    int32_t *state_count;          // [kMaxPend][batch]
    bool shared_row0;              // rows 0 of a prefix's drafts are copies of one another (caller's statement)
    int s_parts;                   // > 1: the sums of Eq. (hik) are left as this many partial sums per row (small batches)
    int e_parts;                   // > 0 (chain schedule): rows marked kExcessPending have their E in this many parts
    int e_coop;                    // != 0 (two-pass schedule): the final-token kernel finds the rows that need E and sums it
    int kseq_ndrafts;              // > 0: the comparison verifier (K-SEQ rule of Section 3.2) on the first kseq_ndrafts drafts
};

// Comparison verifier (Sections 3.1 / 3.2): per row pair the statistics and the root rho (left in lay.s, beta(rho) in
// lay.excess); the scan over positions and the replacement token are a mode of launch_decide_and_sample.
hipError_t launch_kseq_rows(const Problem &p, int ndrafts);

// Schedule "split": statistics kernel, then a second pass for the sums of Eq. (hik).
hipError_t launch_split_main(const Problem &p);
// Parts the two-pass schedule leaves every Eq. (hik) sum in for this problem (1: the sums are complete).
int split_sum_parts(const Problem &p);

// Schedule "chain": one workgroup per (prefix, draft) keeps each row pair on chip between
// the statistics sweep and the Eq. (hik) sweep.  chain_supported() says whether the shape
// fits the kernel's static limits.
bool chain_supported(const Problem &p);
bool chain_preferred(const Problem &p);      // supported, and enough chains for it to beat the two-pass schedule
bool chain_supports_pending(const Problem &p);   // supported, and the whole row pair fits on chip (pending modifications)
hipError_t launch_chain_main(const Problem &p);
// The chain schedule's follow-up kernel: E = nu^2 (s - g) of the rows k_chain handed over (usually none).
hipError_t launch_chain_excess(const Problem &p);
int chain_excess_parts(const Problem &p);    // parts k_chain_excess leaves the cancellation-free sum of a marked row in

// Decision scan (Algorithm 1) and final-token kernels (Eq. (pres) / bonus token).
hipError_t launch_decide_and_sample(const Problem &p);

// One token per row from softmax(logits / T) by inverse CDF with the uniform of Philox slot `slot` of "prefix"
// row; u_out and margin_out receive the uniform and the inverse-CDF margin of every row.
int sample_max_vocab();
hipError_t launch_sample_rows(const void *logits, int rows, int V, int dtype, float c, uint64_t seed, uint64_t offset,
                              uint32_t slot, int32_t *out_tokens, double *u_out, double *margin_out, hipStream_t stream);

// Distribution modification (Algorithm 2); all pointers are device pointers, optional ones may be null.
// `ws` holds modify_workspace_bytes(batch, K, M, bonus) bytes.
size_t modify_workspace_bytes(int batch, int K, int M, int bonus);
hipError_t launch_modify(const void *target, const void *draft, const int32_t *tokens, int K, int M, int bonus, int V,
                         int batch, int dtype, float c, const double *carry, const int32_t *count, float *out_logq,
                         float *out_logp, double *norm_out, int32_t *fallback_out, char *ws, hipStream_t stream);


// Advances a pending modification (carry, count) along the tokens an iteration emitted; `delta` holds batch * M doubles.
hipError_t launch_carry_advance(const void *rows_q, const void *rows_p, const int32_t *tokens, const int32_t *accepted_len,
                                const int32_t *accepted_idx, const int32_t *out_tokens, int K, int M, int bonus, int V,
                                int batch, int dtype, float c, double *carry, int32_t *count, double *delta,
                                hipStream_t stream);

}  // namespace specgbv
