"""GPU <-> oracle parity through the C ABI (needs an MI355X: run with -m gpu).

Every case feeds the same seeded inputs to libspecgbv.so and to the float64 CPU oracle
and compares element by element to the bar written in parity_util.py.
"""
import numpy as np
import pytest

from parity_util import check_case, run_gpu
from specgbv_synth import WORKLOADS, Workload, f32_to_bf16_bits, make_inputs, with_batch

pytestmark = pytest.mark.gpu

ALGOS = ["split", "chain", "auto"]


def chain_takes(V, bf16):
    """The on-chip schedule's static limits: rows of whole 16-byte vectors, at least 3584 of them."""
    pv = 8 if bf16 else 4
    return V % pv == 0 and V // pv >= 3584


def _algo_or_skip(algo, fn, shape=None):
    """Runs fn; a forced chain schedule may refuse a shape only if the shape is outside its stated limits
    (those cases have twins at chain-sized rows in test_gpu_chain_coverage.py).  shape = (V, is_bf16)."""
    import paper_2604_25925_amd as sg
    try:
        return fn()
    except sg.SpecGBVError as e:
        if algo == "chain" and e.status == 2:
            assert shape is None or not chain_takes(*shape), "the chain schedule refused a shape inside its limits"
            pytest.skip("rows too short for the on-chip schedule (covered at chain-sized rows in test_gpu_chain_coverage.py)")
        raise


def _checked(algo, t, d, tok, *args):
    return _algo_or_skip(algo, lambda: check_case(t, d, tok, *args), shape=(t.shape[-1], t.dtype == np.uint16))


@pytest.mark.parametrize("algo", ALGOS)
def test_cfg1_tiny(algo):
    w = WORKLOADS["cfg1"]
    t, d, tok = make_inputs(w, seed=0)
    for off in range(3):
        _checked(algo, t, d, tok, w.temperature, 0, off, algo, "cfg1/off%d" % off)


@pytest.mark.parametrize("algo", ALGOS)
def test_cfg2(algo):
    w = WORKLOADS["cfg2"]
    t, d, tok = make_inputs(w, seed=0)
    _checked(algo, t, d, tok, w.temperature, 0, 0, algo, "cfg2")


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("name", ["cfg3_lo", "cfg3", "cfg3_hi"])
def test_cfg3_reduced_batch(algo, name):
    # same generator and shape as the benchmark configuration, 6 of its 64 prefixes
    w = with_batch(WORKLOADS[name], 6)
    t, d, tok = make_inputs(w, seed=0)
    _checked(algo, t, d, tok, w.temperature, 0, 0, algo, name + "/B6")


@pytest.mark.parametrize("algo", ALGOS)
def test_cfg4_reduced_batch(algo):
    w = with_batch(WORKLOADS["cfg4"], 3)
    t, d, tok = make_inputs(w, seed=0)
    _checked(algo, t, d, tok, w.temperature, 0, 0, algo, "cfg4/B3")


@pytest.mark.parametrize("algo", ALGOS)
def test_cfg5_reduced_batch(algo):
    w = with_batch(WORKLOADS["cfg5"], 2)
    t, d, tok = make_inputs(w, seed=0)
    _checked(algo, t, d, tok, w.temperature, 0, 0, algo, "cfg5/B2")


@pytest.mark.parametrize("B", [1, 2, 3])
@pytest.mark.parametrize("name", ["cfg4", "cfg3"])
def test_small_batches_share_rows_among_workgroups(name, B):
    # with a handful of prefixes the two-pass schedule cuts every row into parts (partial statistics and partial
    # sums of Eq. (hik), combined in part order); batch 1 is the common serving case
    w = with_batch(WORKLOADS[name], B)
    t, d, tok = make_inputs(w, seed=3)
    for off in (0, 1):
        check_case(t, d, tok, w.temperature, 0, off, "auto", "%s/B%d small batch" % (name, B))


def test_cfg4_full_size_sampled_prefixes():
    """The benchmark configuration at full size in the launch configuration bench.py times
    (default schedule); the oracle recomputes 4 of the 32 prefixes."""
    w = WORKLOADS["cfg4"]
    t, d, tok = make_inputs(w, seed=0)
    rep, gpu, _ = check_case(t, d, tok, w.temperature, 0, 0, "auto", "cfg4/full", gpu_slice=[0, 11, 22, 31])
    # properties that hold at any size, on all 32 prefixes
    g = run_gpu(t, d, tok, w.temperature, 0, 0, "auto")
    tau, f, out = g["accepted_len"], g["accepted_draft_idx"], g["out_tokens"]
    assert np.all((tau >= 0) & (tau <= w.L)) and np.all((f == -1) == (tau == 0)) and np.all(f < w.K)
    for b in range(w.batch):
        assert np.array_equal(out[b, :tau[b]], tok[b, max(f[b], 0), :tau[b]])
        assert 0 <= out[b, tau[b]] < w.V and np.all(out[b, tau[b] + 1:] == -1)
    assert np.all((g["h"] >= 0) & (g["h"] <= 1))
    # second run, same counters: bit-identical outputs
    g2 = run_gpu(t, d, tok, w.temperature, 0, 0, "auto")
    for key in ("accepted_len", "accepted_draft_idx", "out_tokens"):
        assert np.array_equal(g[key], g2[key])


# ------------------------------------------------------------ edge cases

def _gauss_case(B, K, L, V, dtype, sigma_t=2.5, sigma_d=0.8, seed=1, T=1.0, head=0):
    w = Workload("edge", B, K, L, V, dtype, sigma_t, sigma_d, head=head, temperature=T)
    return make_inputs(w, seed=seed) + (T,)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("B,K,L,V,dtype", [
    (2, 1, 1, 8, "f32"),          # single draft, single token: token-level rejection sampling
    (3, 1, 6, 515, "f32"),        # single-draft block verification, ragged V (scalar loads)
    (2, 5, 1, 1031, "bf16"),      # L = 1: only whole-block tests, ragged V
    (2, 3, 4, 4104, "bf16"),      # multiple of 8 but not of a segment
    (1, 16, 3, 2048, "f32"),      # exactly one residual segment
    (2, 2, 9, 2056, "bf16"),      # one element group past a segment boundary
    (1, 64, 2, 64, "f32"),        # K at its limit
    (1, 2, 62, 40, "f32"),        # L at its limit
    (5, 4, 3, 70001, "f32"),      # odd V larger than one pass of a workgroup
    (2, 2, 2, 300032, "bf16"),    # more residual segments than the locating workgroup keeps in registers
    (1, 2, 2, 524288, "f32"),
])
def test_shapes_and_ragged_tails(algo, B, K, L, V, dtype):
    t, d, tok, T = _gauss_case(B, K, L, V, dtype)
    for off in (0, 7):
        _checked(algo, t, d, tok, T, 3, off, algo, "edge %s" % ((B, K, L, V, dtype),))


@pytest.mark.parametrize("K,V,dtype", [(1, 32768, "bf16"), (2, 16384, "f32"), (3, 40960, "bf16"), (4, 32768, "bf16"),
                                        (5, 32768, "bf16"), (16, 16384, "f32"), (8, 94208, "bf16"), (3, 65536, "f32"),
                                        (2, 100000, "f32"), (4, 200064, "bf16")])   # rows larger than the on-chip slots
def test_chain_schedule_draft_counts(K, V, dtype):
    # the on-chip schedule has one unrolled variant per common draft count (and a generic one) and
    # three register-slot counts chosen by V; K = 1 is single-draft greedy block verification
    t, d, tok, T = _gauss_case(3, K, 4, V, dtype, seed=20 + K)
    check_case(t, d, tok, T, 4, 1, "chain", "chain K=%d V=%d %s" % (K, V, dtype))


@pytest.mark.parametrize("B,K,L,V,dtype", [(75, 4, 3, 32768, "bf16"), (130, 2, 2, 16384, "f32"), (43, 7, 2, 29696, "bf16")])
def test_chain_schedule_more_chains_than_compute_units(B, K, L, V, dtype):
    # above one chain per compute unit a workgroup walks several chains as one row sequence
    # (300, 260 and 301 chains on 256 compute units: uneven shares, chain boundaries inside the pipeline)
    t, d, tok, T = _gauss_case(B, K, L, V, dtype, seed=33)
    check_case(t, d, tok, T, 6, 2, "chain", "chain %d chains V=%d %s" % (B * K, V, dtype))


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("T", [0.02, 0.1, 0.4, 2.0, 30.0])
def test_temperature(algo, T):
    t, d, tok, _ = _gauss_case(3, 4, 5, 8192, "bf16", T=T)
    _checked(algo, t, d, tok, T, 0, 0, algo, "T=%g" % T)


@pytest.mark.parametrize("algo", ALGOS)
def test_duplicate_drafts_exercise_the_rejected_set(algo):
    # peaked 16-token rows: drafts share prefixes, so blocks recur and H is consulted
    t, d, tok, T = _gauss_case(40, 6, 4, 16, "f32", sigma_t=3.0, sigma_d=1.5, seed=4)
    n_dup = sum(len({tuple(r) for r in tok[b, :, :2]}) < tok.shape[1] for b in range(tok.shape[0]))
    assert n_dup > 10
    rep, gpu, ora = _checked(algo, t, d, tok, T, 9, 0, algo, "duplicates")
    assert np.any(ora["state"] == 2), "no block was skipped through H: case does not test what it should"
    # fully identical drafts: every length is tested once
    t2, d2, tok2 = t.copy(), d.copy(), tok.copy()
    t2[:] = t[:, :1]; d2[:] = d[:, :1]; tok2[:] = tok[:, :1]
    rep, gpu, ora = _checked(algo, t2, d2, tok2, T, 9, 1, algo, "identical drafts")
    assert np.all(gpu["state"][:, 1:, :][ora["state"][:, 1:, :] != 0] == 2)


@pytest.mark.parametrize("algo", ALGOS)
def test_degenerate_residual_draws_from_target_row(algo):
    # p == q: with K >= 2 every residual weight can vanish; the token then comes from q
    rng = np.random.default_rng(2)
    B, K, L, V = 64, 2, 1, 24
    row = rng.normal(0, 1, (B, 1, 1, V)).astype(np.float32)
    t = np.repeat(np.concatenate([row, rng.normal(0, 1, (B, 1, 1, V)).astype(np.float32)], axis=2), K, axis=1)
    d = np.ascontiguousarray(t[:, :, :1])
    tok = rng.integers(0, V, (B, K, L)).astype(np.int32)
    rep, gpu, ora = _checked(algo, t, d, tok, 1.0, 5, 0, algo, "p==q")
    assert ora["fallback"].sum() > 0 and np.array_equal(gpu["fallback"], ora["fallback"])


@pytest.mark.parametrize("algo", ALGOS)
def test_extreme_logits(algo):
    rng = np.random.default_rng(3)
    B, K, L, V = 2, 2, 3, 1024
    t = rng.normal(0, 2, (B, K, L + 1, V)).astype(np.float32)
    t[0] -= 900.0                      # all far below zero
    t[1] += 700.0                      # all far above zero
    t[1, 0, 1, 5] += 60.0              # one dominant token
    d = (t[:, :, :L] + rng.normal(0, 1, (B, K, L, V))).astype(np.float32)
    tok = rng.integers(0, V, (B, K, L)).astype(np.int32)
    tok[1, 0, 1] = 5
    _checked(algo, t, d, tok, 1.0, 0, 0, algo, "extreme f32")
    tb, db = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    _checked(algo, tb, db, tok, 0.7, 0, 0, algo, "extreme bf16")


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("dtype,V", [("f32", 3000), ("bf16", 32768)])
def test_masked_logits_minus_infinity(algo, dtype, V):
    # vocabulary masks: -inf in both models (padded tail), in the target only and in the draft only
    # (never at a drafted token's draft logit); a masked entry has probability 0 and weight 0
    t, d, tok, T = _gauss_case(3, 4, 4, V, "f32", seed=11)
    rng = np.random.default_rng(12)
    t[..., V - 200:] = -np.inf
    d[..., V - 200:] = -np.inf
    only_t = rng.integers(0, V - 200, 300)
    only_d = rng.integers(0, V - 200, 300)
    t[..., only_t] = -np.inf
    d[..., only_d] = -np.inf
    B, K, L = tok.shape
    for b in range(B):
        for k in range(K):
            for r in range(L):
                # the drafted token must have positive draft probability: redraw onto an unmasked entry
                while not np.isfinite(d[b, k, r, tok[b, k, r]]) or not np.isfinite(t[b, k, r, tok[b, k, r]]):
                    tok[b, k, r] = rng.integers(0, V - 200)
    # one drafted token that the target forbids outright: its block and every longer one have nu = 0
    t[1, 2, 1, tok[1, 2, 1]] = -np.inf
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    for off in (0, 1):
        rep, gpu, ora = _checked(algo, t, d, tok, T, 2, off, algo, "masked %s" % dtype)
        assert np.all(ora["h"][1, 2, 1:] == 0.0) and np.all(gpu["h"][1, 2, 1:] == 0.0)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("T", [0.8, 0.56])
def test_forbidden_tokens_at_other_temperatures(algo, T):
    # Drafted tokens the target gives probability zero (nu = 0 from there on) and target-only tokens (p = 0, so the
    # ratio carried to the next iteration is infinite when one is drawn), at temperatures whose float32 scale is
    # rounded down (0.56) and up (0.8): the first-order correction for that rounding must leave infinities alone.
    t, d, tok, _ = _gauss_case(6, 3, 4, 32768, "f32", seed=21, T=T)
    rng = np.random.default_rng(22)
    V = t.shape[-1]
    d[..., rng.integers(0, V, V // 3)] = -np.inf           # a third of the vocabulary unknown to the draft model
    B, K, L = tok.shape
    for b in range(B):
        for k in range(K):
            for r in range(L):
                while not np.isfinite(d[b, k, r, tok[b, k, r]]):
                    tok[b, k, r] = rng.integers(0, V)
    for b in range(B):
        t[b, b % K, 1 + b % (L - 1), tok[b, b % K, 1 + b % (L - 1)]] = -np.inf
    t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    seen_inf = False
    for off in range(4):
        rep, gpu, ora = _checked(algo, t, d, tok, T, 5, off, algo, "forbidden tokens T=%g" % T)
        assert np.array_equal(np.isneginf(ora["log_nu"]), np.isneginf(gpu["log_nu"])) and np.isneginf(ora["log_nu"]).any()
        seen_inf = seen_inf or bool(np.isposinf(ora["carry_log_nu"]).any())
        assert np.array_equal(np.isposinf(ora["carry_log_nu"]), np.isposinf(gpu["carry_log_nu"]))
    assert seen_inf                                          # some final token was one the draft model cannot produce


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_whole_segments_masked_in_every_row(algo, dtype):
    # vocabulary padding longer than a 512-entry residual segment, masked with -inf in both models: a segment
    # without a finite entry must weigh nothing, in the residual rows and in the bonus row alike (prefix 0 has
    # identical models: either its whole block is accepted or every residual weight vanishes and the token comes
    # from the target row; at every offset some prefix accepts a whole block and draws from the bonus row).
    t, d, tok, T = _gauss_case(4, 3, 3, 16384, "f32", seed=17)
    V = t.shape[-1]
    rng = np.random.default_rng(18)
    d[0] = t[0, :, :3]
    for a in (t, d):
        a[..., :1100] = -np.inf
        a[..., 6000:7700] = -np.inf
        a[..., V - 2048:] = -np.inf
    t[1] -= 500.0                                  # both models far from zero, by the same offset
    d[1] -= 500.0
    B, K, L = tok.shape
    for b in range(B):
        for k in range(K):
            for r in range(L):
                while not np.isfinite(d[b, k, r, tok[b, k, r]]):
                    tok[b, k, r] = rng.integers(1100, 6000)
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    for off in (0, 1, 2):
        rep, gpu, ora = _checked(algo, t, d, tok, T, 3, off, algo, "masked segments %s" % dtype)
        assert np.any(ora["accepted_len"] == L), "no prefix reaches the bonus row: case does not test what it should"
        y = gpu["out_tokens"][np.arange(B), gpu["accepted_len"]]
        assert np.all(((y >= 1100) & (y < 6000)) | ((y >= 7700) & (y < V - 2048)))


def test_plain_entry_point_matches_ex_and_offsets_differ():
    w = with_batch(WORKLOADS["cfg2"], 4)
    t, d, tok = make_inputs(w, seed=2)
    a = run_gpu(t, d, tok, 1.0, 11, 5, plain=True)
    b = run_gpu(t, d, tok, 1.0, 11, 5, algo="auto")
    for key in a:
        assert np.array_equal(a[key], b[key], equal_nan=True), key
    c = run_gpu(t, d, tok, 1.0, 11, 6, plain=True)
    assert not np.array_equal(a["eta"], c["eta"])
    assert np.array_equal(a["h"], c["h"])


def test_empty_batch_and_argument_errors_on_device():
    import torch
    import paper_2604_25925_amd as sg
    t = torch.zeros((0, 2, 3, 64), device="cuda")
    d = torch.zeros((0, 2, 2, 64), device="cuda")
    tok = torch.zeros((0, 2, 2), dtype=torch.int32, device="cuda")
    a, f, o, _ = sg.specgbv_verify(t, d, tok, 1.0, 0, 0)
    assert a.numel() == 0 and o.shape == (0, 3)
    t = torch.zeros((1, 2, 3, 64), device="cuda")
    d = torch.zeros((1, 2, 2, 64), device="cuda")
    tok = torch.zeros((1, 2, 2), dtype=torch.int32, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sg.SpecGBVError) as ei:
        sg.specgbv_verify(t, d, tok, 1.0, 0, 0, workspace=small)
    assert ei.value.status == 3
    with pytest.raises(sg.SpecGBVError) as ei:
        sg.specgbv_verify(t, d, tok, float("nan"), 0, 0)
    assert ei.value.status == 1
