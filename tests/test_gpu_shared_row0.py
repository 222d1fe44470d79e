"""Chain schedule with the caller's statement that a prefix's drafts share their rows 0 (needs an MI355X).

In Algorithm 3 the K drafts of an iteration extend one prefix, so position 0 of every draft sees the same
two distributions; with `shared_row0` the library reduces those rows once per prefix (a small kernel of
its own) and every chain starts at row 1.  The oracle knows nothing of this: it reads every draft's own
rows, which the generator makes copies of one another, so the comparison is the ordinary parity check.
"""
import numpy as np
import pytest

from parity_util import check_case, run_gpu
from specgbv_synth import WORKLOADS, Workload, f32_to_bf16_bits, make_inputs, with_batch

pytestmark = pytest.mark.gpu


def _shared(t, d):
    return np.array_equal(t[:, :, 0], np.broadcast_to(t[:, :1, 0], t[:, :, 0].shape)) and \
        np.array_equal(d[:, :, 0], np.broadcast_to(d[:, :1, 0], d[:, :, 0].shape))


def _gauss_case(B, K, L, V, dtype, sigma_t=2.5, sigma_d=0.8, seed=1, T=1.0, head=0):
    w = Workload("edge", B, K, L, V, dtype, sigma_t, sigma_d, head=head, temperature=T)
    t, d, tok = make_inputs(w, seed=seed)
    assert _shared(t, d), "the generator is expected to give a prefix's drafts the same rows 0"
    return t, d, tok, T


@pytest.mark.parametrize("name,B", [("cfg2", 8), ("cfg3", 5), ("cfg4", 3), ("cfg5", 2)])
def test_benchmark_configurations(name, B):
    w = with_batch(WORKLOADS[name], B)
    t, d, tok = make_inputs(w, seed=0)
    assert _shared(t, d)
    check_case(t, d, tok, w.temperature, 0, 0, "chain", "%s/B%d shared row 0" % (name, B), shared_row0=True)


def test_cfg4_full_size_sampled_prefixes():
    # the launch configuration bench.py times by default; the oracle checks four of the 32 prefixes
    w = WORKLOADS["cfg4"]
    t, d, tok = make_inputs(w, seed=0)
    rep, gpu, _ = check_case(t, d, tok, w.temperature, 0, 0, "auto", "cfg4/full shared row 0", gpu_slice=[0, 9, 20, 31],
                             shared_row0=True)


@pytest.mark.parametrize("K,L,V,dtype", [(1, 4, 32768, "bf16"), (2, 2, 16384, "f32"), (3, 5, 40960, "bf16"),
                                          (8, 3, 94208, "bf16"), (16, 2, 16384, "f32"), (5, 9, 32768, "bf16"),
                                          (4, 3, 200064, "bf16"), (2, 4, 100000, "f32")])
def test_draft_counts_and_lengths(K, L, V, dtype):
    # L = 2: a chain is a single row; rows larger than the on-chip slots; every register-slot variant
    t, d, tok, T = _gauss_case(3, K, L, V, dtype, seed=40 + K)
    rep, gpu, ora = check_case(t, d, tok, T, 4, 1, "chain", "shared row 0 K=%d L=%d V=%d %s" % (K, L, V, dtype),
                               shared_row0=True)
    # every draft of a prefix gets the same bits for position 0
    assert np.array_equal(gpu["lse_q"][:, :, 0], np.broadcast_to(gpu["lse_q"][:, :1, 0], gpu["lse_q"][:, :, 0].shape))
    assert np.array_equal(gpu["lse_p"][:, :, 0], np.broadcast_to(gpu["lse_p"][:, :1, 0], gpu["lse_p"][:, :, 0].shape))


@pytest.mark.parametrize("B,K,L,V,dtype", [(75, 4, 3, 32768, "bf16"), (130, 2, 2, 16384, "f32"), (43, 7, 4, 29696, "bf16")])
def test_more_chains_than_compute_units(B, K, L, V, dtype):
    # a workgroup walks several chains as one row sequence; each chain's position 0 comes from its own prefix
    t, d, tok, T = _gauss_case(B, K, L, V, dtype, seed=35)
    check_case(t, d, tok, T, 6, 2, "chain", "shared row 0, %d chains V=%d %s" % (B * K, V, dtype), shared_row0=True)


def test_single_token_blocks_ignore_the_hint():
    # L = 1: a chain has no row beyond position 0, the rows are read the ordinary way
    t, d, tok, T = _gauss_case(4, 3, 1, 16384, "f32", seed=8)
    check_case(t, d, tok, T, 1, 0, "chain", "shared row 0, L=1", shared_row0=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_masked_slices_and_extreme_offsets(dtype):
    # a whole slice of the shared rows masked out (its partial sum is empty), the rest far from zero
    t, d, tok, T = _gauss_case(3, 4, 3, 32768, "f32", seed=13)
    V = t.shape[-1]
    t[..., : V // 16 + 40] = -np.inf              # first slice of every row, and a little of the second
    d[..., : V // 16 + 40] = -np.inf
    t[0] -= 800.0                                 # both models far from zero, by the same offset
    d[0] -= 800.0
    t[1] += 600.0
    d[1] += 600.0
    rng = np.random.default_rng(14)
    B, K, L = tok.shape
    for b in range(B):
        for k in range(K):
            for r in range(L):
                while not np.isfinite(d[b, k, r, tok[b, k, r]]):
                    tok[b, k, r] = rng.integers(V // 16 + 40, V)
    assert _shared(t, d)
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    check_case(t, d, tok, T, 2, 0, "chain", "shared row 0, masked slice %s" % dtype, shared_row0=True)


def test_other_schedules_ignore_the_hint():
    t, d, tok, T = _gauss_case(3, 4, 4, 16384, "bf16", seed=21)
    a = run_gpu(t, d, tok, T, 5, 0, algo="split")
    b = run_gpu(t, d, tok, T, 5, 0, algo="split", shared_row0=True)
    for key in a:
        assert np.array_equal(a[key], b[key], equal_nan=True), key


def test_rows_of_draft_0_stand_for_every_draft():
    # rows 0 that differ (the caller's statement is false): position 0 of every draft is then taken from draft 0's
    # rows, i.e. the result is that of the inputs with draft 0's rows 0 copied to every draft
    t, d, tok, T = _gauss_case(3, 4, 3, 16384, "f32", seed=22)
    rng = np.random.default_rng(23)
    t2, d2 = t.copy(), d.copy()
    t2[:, 1:, 0] += rng.normal(0, 1, t2[:, 1:, 0].shape).astype(np.float32)
    d2[:, 1:, 0] += rng.normal(0, 1, d2[:, 1:, 0].shape).astype(np.float32)
    a = run_gpu(t, d, tok, T, 5, 0, algo="chain", shared_row0=True)
    b = run_gpu(t2, d2, tok, T, 5, 0, algo="chain", shared_row0=True)
    for key in ("accepted_len", "accepted_draft_idx", "out_tokens", "lse_q", "lse_p", "log_nu", "h"):
        assert np.array_equal(a[key], b[key], equal_nan=True), key
