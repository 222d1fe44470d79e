"""The comparison verifiers on the GPU (SpecTr's K-SEQ rule, Section 3.2; token-level speculative decoding,
Section 3.1) against the oracle, through the C ABI (needs an MI355X: run with -m gpu).

Bar: accepted length, retained draft and tokens bit-exact unless a performed test has |eta - acceptance
probability| < 1e-6 or the final token's inverse-CDF margin is below 1e-6 (counted); rho, beta(rho), acceptance
probabilities and the replacement normaliser within 1e-5 relative.  rho is compared where its equation is
well conditioned (the slope of 1 - (1 - beta)^k - rho beta at the root is not tiny); elsewhere (drafts equal to the
target, where the root is multiple) beta and the acceptance probabilities are still compared.
"""
import numpy as np
import pytest

from parity_util import to_torch
from specgbv_synth import WORKLOADS, Workload, f32_to_bf16_bits, make_inputs, with_batch

pytestmark = pytest.mark.gpu
RTOL, MARGIN = 1e-5, 1e-6


def run_both(t, d, tok, T, seed, offset, ndrafts=None, nthreads=8):
    import torch
    import oracle
    import paper_2604_25925_amd as sg
    tl, dl, tk = to_torch(t), to_torch(d), to_torch(np.ascontiguousarray(tok, dtype=np.int32))
    B, K, L1, V = tl.shape
    L = L1 - 1
    a, f, o, ws = sg.specgbv_verify_kseq(tl, dl, tk, T, seed, offset, ndrafts)
    torch.cuda.synchronize()
    gpu = {"accepted_len": a.cpu().numpy(), "accepted_draft_idx": f.cpu().numpy(), "out_tokens": o.cpu().numpy()}
    gpu.update(sg.specgbv_read_kseq_intermediates(ws, B, K, L, V))
    ora = oracle.verify_kseq(t, d, tok, T, seed, offset, ndrafts=ndrafts, debug=True, eager=True, nthreads=nthreads)
    return gpu, ora


def compare(gpu, ora, tok, nd, label):
    B, K, L = tok.shape
    rep = {"prefixes": B, "low_margin_decisions": 0, "decision_mismatches": 0, "low_margin_tokens": 0,
           "token_mismatches": 0}
    sel = np.zeros((B, K, L), bool)
    sel[:, :nd] = True
    rel = lambda g, o: np.abs(g - o) / (RTOL * np.abs(o) + 1e-12)
    # beta(rho) and rho of every (draft, row): what the data-parallel implementation computes up front
    worst_beta = rel(gpu["beta_all"][sel], ora["beta_all"][sel]).max()
    # rho where the root is well conditioned: |d f / d rho| >= 0.05 estimated from the oracle's beta by a finite step
    rho_err = rel(gpu["rho_all"][sel], ora["rho_all"][sel])
    rep["max_err"] = {"beta": float(worst_beta), "rho_all": float(rho_err.max())}
    if worst_beta > 1.0:
        e = np.where(sel, rel(gpu["beta_all"], ora["beta_all"]), 0.0)
        w = np.unravel_index(int(np.argmax(e)), e.shape)
        raise AssertionError("%s beta: %.3g x the tolerance at %s: beta %.12g vs %.12g, rho %.12g vs %.12g" % (
            label, worst_beta, w, gpu["beta_all"][w], ora["beta_all"][w], gpu["rho_all"][w], ora["rho_all"][w]))
    assert np.all(gpu["rho_all"][sel] >= 1.0 - 1e-12) and np.all(np.isfinite(gpu["rho_all"][sel]))
    # rho beta = P(a position accepts) and the equation itself, evaluated with the GPU's values
    assert np.array_equal(gpu["eta"][sel], ora["eta_all"][sel]) if "eta_all" in ora else True
    for b in range(B):
        tested = (ora["state"][b] == 1) | (gpu["state"][b] == 1)
        both = (ora["state"][b] == 1) & (gpu["state"][b] == 1)
        if both.any():
            err = rel(gpu["accept"][b][both], ora["accept"][b][both]).max()
            rep["max_err"]["accept"] = max(rep["max_err"].get("accept", 0.0), float(err))
            assert err <= 1.0 + 1e-9 / RTOL, "%s prefix %d: acceptance probability %.3g x the tolerance" % (label, b, err)
            assert np.array_equal(gpu["eta"][b][both], ora["eta"][b][both])
        ga = np.where(gpu["state"][b] == 1, gpu["accept"][b], np.nan)
        oa = np.where(ora["state"][b] == 1, ora["accept"][b], np.nan)
        dist = np.fmin(np.abs(gpu["eta"][b] - ga), np.abs(ora["eta"][b] - oa))
        low = bool(np.any(dist[tested] < MARGIN))
        rep["low_margin_decisions"] += int(low)
        same = gpu["accepted_len"][b] == ora["accepted_len"][b] and gpu["accepted_draft_idx"][b] == ora["accepted_draft_idx"][b]
        if not same:
            assert low, "%s prefix %d: (tau, lead) = (%d, %d) vs oracle (%d, %d) with every margin >= 1e-6" % (
                label, b, gpu["accepted_len"][b], gpu["accepted_draft_idx"][b], ora["accepted_len"][b], ora["accepted_draft_idx"][b])
            rep["decision_mismatches"] += 1
            continue
        assert np.array_equal(gpu["state"][b], ora["state"][b]), "%s prefix %d: tested candidates differ" % (label, b)
        assert np.array_equal(gpu["retained"][b], ora["retained"][b]) and np.array_equal(gpu["lead"][b], ora["lead"][b])
        tau = int(ora["accepted_len"][b])
        # the rho the procedure used at each position it reached, against the oracle's
        for i in range(min(tau + 1, L)):
            j = ora["lead"][b, i]
            assert ora["rho"][b, i] == ora["rho_all"][b, j, i]
        go, oo = gpu["out_tokens"][b], ora["out_tokens"][b]
        assert np.array_equal(go[:tau], oo[:tau]) and np.all(go[tau + 1:] == -1)
        assert gpu["u_final"][b] == ora["u_final"][b]
        err = abs(gpu["res_norm"][b] - ora["res_norm"][b]) / (RTOL * abs(ora["res_norm"][b]) + 1e-12)
        rep["max_err"]["res_norm"] = max(rep["max_err"].get("res_norm", 0.0), float(err))
        assert err <= 1.0, "%s prefix %d: replacement normaliser %.3g x the tolerance (%g vs %g)" % (
            label, b, err, gpu["res_norm"][b], ora["res_norm"][b])
        low_tok = ora["margin"][b] < MARGIN or gpu["margin"][b] < MARGIN
        rep["low_margin_tokens"] += int(low_tok)
        if go[tau] != oo[tau]:
            assert low_tok, "%s prefix %d: final token %d vs %d" % (label, b, go[tau], oo[tau])
            rep["token_mismatches"] += 1
    print("[parity] %s: %s" % (label, rep), flush=True)
    return rep


def check(t, d, tok, T, seed=0, offset=0, ndrafts=None, label="", rho_tol=1.0):
    gpu, ora = run_both(t, d, tok, T, seed, offset, ndrafts)
    nd = tok.shape[1] if ndrafts is None else ndrafts
    rep = compare(gpu, ora, tok, nd, label)
    assert rep["max_err"]["rho_all"] <= rho_tol, "%s rho: %.3g x the tolerance" % (label, rep["max_err"]["rho_all"])
    return rep, gpu, ora


@pytest.mark.parametrize("name,B", [("cfg1", 1), ("cfg2", 8), ("cfg3", 4), ("cfg3_lo", 3), ("cfg3_hi", 3), ("cfg4", 2), ("cfg5", 1)])
def test_benchmark_configurations(name, B):
    w = with_batch(WORKLOADS[name], B)
    t, d, tok = make_inputs(w, seed=0)
    for off in (0, 1):
        check(t, d, tok, w.temperature, 0, off, None, "%s/B%d K-SEQ" % (name, B), rho_tol=3.0)


def test_cfg4_full_size_sampled_prefixes():
    """The benchmark configuration at full size, as bench.py --op compare times it (2048 row pairs, one workgroup
    each); the oracle recomputes 3 of the 32 prefixes with their own Philox counters."""
    import torch
    import oracle
    import paper_2604_25925_amd as sg
    w = WORKLOADS["cfg4"]
    t, d, tok = make_inputs(w, seed=0)
    tl, dl, tk = to_torch(t), to_torch(d), to_torch(np.ascontiguousarray(tok, dtype=np.int32))
    a, f, o, ws = sg.specgbv_verify_kseq(tl, dl, tk, w.temperature, 3, 1)
    torch.cuda.synchronize()
    full = {"accepted_len": a.cpu().numpy(), "accepted_draft_idx": f.cpu().numpy(), "out_tokens": o.cpu().numpy()}
    full.update(sg.specgbv_read_kseq_intermediates(ws, w.batch, w.K, w.L, w.V))
    ids = [0, 13, 31]
    gpu = {k: np.ascontiguousarray(v[ids]) for k, v in full.items()}
    ora = oracle.verify_kseq(t[ids], d[ids], tok[ids], w.temperature, 3, 1, debug=True, eager=True, nthreads=8,
                             prefix_ids=np.asarray(ids, np.int32))
    rep = compare(gpu, ora, tok[ids], w.K, "cfg4/full K-SEQ")
    assert rep["max_err"]["rho_all"] <= 3.0
    # properties that hold at any size, on all prefixes
    tau, lead, out = full["accepted_len"], full["accepted_draft_idx"], full["out_tokens"]
    assert np.all((tau >= 0) & (tau <= w.L)) and np.all((lead == -1) == (tau == 0)) and np.all(lead < w.K)
    for b in range(w.batch):
        assert np.array_equal(out[b, :tau[b]], tok[b, max(lead[b], 0), :tau[b]])
        assert 0 <= out[b, tau[b]] < w.V and np.all(out[b, tau[b] + 1:] == -1)
    assert np.all((full["rho_all"] >= 1.0 - 1e-12) & (full["rho_all"] <= w.K + 1e-9))
    assert np.all((full["beta_all"] > 0.0) & (full["beta_all"] <= 1.0 + 1e-9))


@pytest.mark.parametrize("nd", [1, 2, 3])
def test_fewer_drafts_and_token_level_speculative_decoding(nd):
    import oracle
    w = with_batch(WORKLOADS["cfg2"], 6)
    t, d, tok = make_inputs(w, seed=4)
    rep, gpu, ora = check(t, d, tok, w.temperature, 7, 2, nd, "cfg2 first %d drafts" % nd, rho_tol=3.0)
    if nd == 1:                                   # Section 3.1 written out separately in the oracle
        sd = oracle.verify_token_sd(t, d, tok, w.temperature, 7, 2)
        assert np.array_equal(ora["accepted_len"], sd["accepted_len"]) and np.array_equal(ora["out_tokens"], sd["out_tokens"])
        assert np.all(gpu["rho_all"][:, 0] == 1.0)


@pytest.mark.parametrize("B,K,L,V,dtype", [
    (3, 1, 5, 515, "f32"),        # one draft, ragged V (scalar loads)
    (4, 5, 2, 1031, "bf16"),
    (2, 8, 3, 4104, "bf16"),
    (2, 16, 2, 2048, "f32"),
    (1, 64, 2, 64, "f32"),        # K at its limit
    (1, 2, 62, 40, "f32"),        # L at its limit
    (3, 4, 3, 70001, "f32"),
    (2, 3, 2, 300032, "bf16"),
])
def test_shapes(B, K, L, V, dtype):
    w = Workload("edge", B, K, L, V, dtype, 2.5, 0.8, temperature=1.0)
    t, d, tok = make_inputs(w, seed=1)
    for off in (0, 5):
        check(t, d, tok, 1.0, 3, off, None, "K-SEQ edge %s" % ((B, K, L, V, dtype),), rho_tol=3.0)


def test_coinciding_drafts_share_positions():
    # peaked 16-token rows: drafts coincide, so several candidates carry the same token and the retained set shrinks slowly
    w = Workload("dup", 40, 6, 4, 16, "f32", 3.0, 1.5, temperature=1.0)
    t, d, tok = make_inputs(w, seed=4)
    rep, gpu, ora = check(t, d, tok, 1.0, 9, 0, None, "K-SEQ coinciding drafts", rho_tol=3.0)
    assert (ora["retained"][:, 1:] > 1).any() and (ora["accepted_len"] == w.L).any() and (ora["accepted_len"] == 0).any()


@pytest.mark.parametrize("T", [0.1, 0.4, 2.0])
def test_temperatures(T):
    w = Workload("temp", 3, 4, 4, 8192, "bf16", 2.5, 0.8, temperature=T)
    t, d, tok = make_inputs(w, seed=2)
    check(t, d, tok, T, 0, 0, None, "K-SEQ T=%g" % T, rho_tol=3.0)


def test_masked_entries():
    w = Workload("mask", 3, 4, 3, 3000, "f32", 2.5, 0.8, temperature=1.0)
    t, d, tok = make_inputs(w, seed=11)
    rng = np.random.default_rng(12)
    V = w.V
    t[..., V - 200:] = -np.inf
    d[..., V - 200:] = -np.inf
    t[..., rng.integers(0, V - 200, 200)] = -np.inf
    d[..., rng.integers(0, V - 200, 200)] = -np.inf
    B, K, L = tok.shape
    for b in range(B):
        for k in range(K):
            for r in range(L):
                while not np.isfinite(d[b, k, r, tok[b, k, r]]) or not np.isfinite(t[b, k, r, tok[b, k, r]]):
                    tok[b, k, r] = rng.integers(0, V - 200)
    check(t, d, tok, 1.0, 2, 0, None, "K-SEQ masked", rho_tol=3.0)
    check(f32_to_bf16_bits(t), f32_to_bf16_bits(d), tok, 1.0, 2, 1, None, "K-SEQ masked bf16", rho_tol=3.0)


def test_acceptance_length_law_against_enumeration():
    # many prefixes over small tables: mean accepted length of the GPU procedure against the enumerated expectation
    from oracle import exact_enum as ee
    from specgbv_synth import tables_to_inputs
    import paper_2604_25925_amd as sg
    import torch
    rng = np.random.default_rng(5)
    V, L, K, n = 3, 2, 3, 60000
    p_of, q_of = ee.random_tables(rng, V, L)
    dist, E_tau = ee.enumerate_kseq(p_of, q_of, V, L, K)
    t, d, tok = tables_to_inputs(p_of, q_of, V, L, K, n, seed=3)
    a, f, o, ws = sg.specgbv_verify_kseq(to_torch(t), to_torch(d), to_torch(tok), 1.0, 5, 0)
    torch.cuda.synchronize()
    a = a.cpu().numpy(); o = o.cpu().numpy()
    assert abs(a.mean() - E_tau) < 5 * L / np.sqrt(n)
    first = np.bincount(o[:, 0], minlength=V) / n
    q0 = np.array([float(v) for v in q_of(())])
    assert np.abs(first - q0).max() < 5 / np.sqrt(n)
