"""Pins for the oracle's comparison verifiers (no GPU): token-level speculative decoding (Section 3.1) and
SpecTr's K-SEQ rule (Section 3.2).

What fixes them from outside the oracle:
  * the defining equation of rho, 1 - (1 - beta)^k = rho beta, and a hand-solved quadratic case;
  * k = 1 gives rho = 1 and the procedure of Section 3.1, which is written out separately;
  * SpecTr is distribution-preserving: by brute-force enumeration the emitted tokens follow the target for every
    K -- and do NOT if rho is always solved for k = K instead of the number of drafts still retained, which is
    how the reading taken at later positions is justified;
  * more drafts never shorten the accepted length (closed form at L = 1: 1 - (1 - beta)^K);
  * the C procedure's Monte-Carlo law against the enumerated law (chi-squared).
"""
import itertools
import math
from fractions import Fraction as F

import numpy as np
import pytest
from scipy.stats import chi2

import oracle
from oracle import exact_enum as ee
from specgbv_synth import tables_to_inputs


def _rows(rng, V, conc=0.5):
    q = rng.dirichlet(np.ones(V) * conc) + 1e-12
    p = rng.dirichlet(np.ones(V) * conc) + 1e-12
    return q / q.sum(), p / p.sum()


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8, 16])
def test_rho_solves_its_equation(k):
    rng = np.random.default_rng(k)
    for _ in range(20):
        q, p = _rows(rng, 64)
        rho = oracle.kseq_rho(np.log(q), np.log(p), k)
        assert 1.0 <= rho <= k
        beta = np.minimum(p, q / rho).sum()                 # beta(rho), typed from its definition
        assert abs(oracle.kseq_beta(np.log(q), np.log(p), rho) - beta) < 1e-14
        assert abs(1 - (1 - beta) ** k - rho * beta) < 1e-12
    # p == q: beta(rho) = 1/rho and the equation reads (1 - 1/rho)^k = 0, a k-fold root at rho = 1; the rounding of
    # beta (1e-16) moves a k-fold root by its k-th root, which is as close as any float64 solver can get
    assert abs(oracle.kseq_rho(np.log(q), np.log(q), k) - 1.0) <= 2 * 1e-16 ** (1.0 / max(k, 1))


def test_rho_hand_solved_quadratic():
    # V = 2, k = 2, p = (1/2, 1/2), q = (4/5, 1/5).  For rho in [1, 8/5]: min{p0, q0/rho} = 1/2 and
    # min{p1, q1/rho} = 1/(5 rho), so beta = 1/2 + 1/(5 rho); with k = 2 the equation reduces to beta = 2 - rho,
    # i.e. 10 rho^2 - 15 rho + 2 = 0, whose root in the range is (15 + sqrt(145)) / 20.
    rho = oracle.kseq_rho(np.log([0.8, 0.2]), np.log([0.5, 0.5]), 2)
    assert abs(rho - (15 + math.sqrt(145)) / 20) < 1e-13
    assert 1 < rho < 1.6


def test_single_draft_is_token_level_speculative_decoding():
    rng = np.random.default_rng(5)
    B, K, L, V = 400, 3, 4, 12
    t = rng.normal(0, 1.5, (B, K, L + 1, V)).astype(np.float32)
    d = (t[:, :, :L] + rng.normal(0, 1.0, (B, K, L, V))).astype(np.float32)
    tok = rng.integers(0, V, (B, K, L)).astype(np.int32)
    a = oracle.verify_kseq(t, d, tok, 0.9, 3, 1, ndrafts=1, debug=True)
    b = oracle.verify_token_sd(t, d, tok, 0.9, 3, 1)
    assert np.array_equal(a["accepted_len"], b["accepted_len"]) and np.array_equal(a["out_tokens"], b["out_tokens"])
    assert np.all(a["rho"][a["retained"] > 0] == 1.0)
    assert len(set(a["accepted_len"].tolist())) >= 4
    # acceptance probability min{1, q/p} of Section 3.1 on the tested entries of draft 0
    lq = t[:, 0, :L] / 0.9 - np.log(np.exp(t[:, 0, :L].astype(np.float64) / np.float32(0.9)).sum(-1, keepdims=True))
    lp = d[:, 0] / 0.9 - np.log(np.exp(d[:, 0].astype(np.float64) / np.float32(0.9)).sum(-1, keepdims=True))
    idx = tok[:, 0, :, None]
    alpha = np.minimum(1.0, np.exp(np.take_along_axis(lq, idx, -1) - np.take_along_axis(lp, idx, -1)))[..., 0]
    tested = a["state"][:, 0] == 1
    assert np.allclose(a["accept"][:, 0][tested], alpha[tested], rtol=1e-6)


def _first_token_law(dist, V):
    out = np.zeros(V)
    for toks, pr in dist.items():
        out[toks[0]] += pr
    return out


@pytest.mark.parametrize("V,L,K", [(2, 1, 1), (2, 1, 2), (3, 1, 3), (2, 1, 5), (2, 2, 2), (3, 2, 2), (2, 2, 3), (2, 3, 2)])
def test_kseq_preserves_the_target_distribution(V, L, K):
    """Enumerated law of the emitted tokens: the first token follows q(.|prefix), and given that a first token a
    was ACCEPTED the second emitted token follows q(.|a) (an accepted token is always followed by another one)."""
    rng = np.random.default_rng(17 * V + 5 * L + K)
    p_of, q_of = ee.random_tables(rng, V, L)
    dist, E_tau = ee.enumerate_kseq(p_of, q_of, V, L, K)
    assert abs(sum(dist.values()) - 1) < 1e-12
    q0 = np.array([float(v) for v in q_of(())])
    assert np.abs(_first_token_law(dist, V) - q0).max() < 1e-12
    if L >= 2:
        for a in range(V):
            mass = sum(pr for toks, pr in dist.items() if len(toks) >= 2 and toks[0] == a)
            for b2 in range(V):
                got = sum(pr for toks, pr in dist.items() if len(toks) >= 2 and toks[:2] == (a, b2))
                assert abs(got / mass - float(q_of((a,))[b2])) < 1e-11
    assert 0 <= E_tau <= L


def test_retained_count_reading_is_the_one_that_preserves_the_target():
    # V = 2, L = 2, K = 3: with rho solved for k = K at the second position too, the second token's law is off
    rng = np.random.default_rng(3)
    worst_ok, worst_bad = 0.0, 0.0
    for _ in range(5):
        p_of, q_of = ee.random_tables(rng, 2, 2)
        for reading, store in ((True, "ok"), (False, "bad")):
            dist, _ = ee.enumerate_kseq(p_of, q_of, 2, 2, 3, retained_reading=reading)
            err = 0.0
            for a in range(2):
                mass = sum(pr for toks, pr in dist.items() if len(toks) >= 2 and toks[0] == a)
                for b2 in range(2):
                    got = sum(pr for toks, pr in dist.items() if len(toks) >= 2 and toks[:2] == (a, b2))
                    err = max(err, abs(got / mass - float(q_of((a,))[b2])))
            if store == "ok":
                worst_ok = max(worst_ok, err)
            else:
                worst_bad = max(worst_bad, err)
    assert worst_ok < 1e-11
    assert worst_bad > 1e-3


def test_more_drafts_accept_at_least_as_much_at_one_position():
    # L = 1: a candidate is accepted with probability beta(rho_K), so P(accept) = 1 - (1 - beta)^K = rho beta
    rng = np.random.default_rng(9)
    p_of, q_of = ee.random_tables(rng, 3, 1)
    prev = -1.0
    for K in (1, 2, 3, 4):
        dist, E_tau = ee.enumerate_kseq(p_of, q_of, 3, 1, K)
        p = [float(v) for v in p_of(())]; q = [float(v) for v in q_of(())]
        rho = ee.kseq_rho_float(p, q, K)
        beta = sum(min(px, qx / rho) for px, qx in zip(p, q))
        assert abs(E_tau - rho * beta) < 1e-12 and abs(E_tau - (1 - (1 - beta) ** K)) < 1e-12
        assert E_tau >= prev - 1e-12
        prev = E_tau
    # K = 1: the acceptance probability of token-level speculative decoding, sum_x min{p, q}
    assert abs(ee.enumerate_kseq(p_of, q_of, 3, 1, 1)[1] - sum(min(a, b) for a, b in zip(p, q))) < 1e-12


@pytest.mark.parametrize("V,L,K,n", [(3, 2, 3, 200000), (2, 3, 2, 200000), (4, 1, 4, 150000)])
def test_c_procedure_follows_the_enumerated_law(V, L, K, n):
    rng = np.random.default_rng(100 + V + L + K)
    p_of, q_of = ee.random_tables(rng, V, L)
    dist, E_tau = ee.enumerate_kseq(p_of, q_of, V, L, K)
    t, d, tok = tables_to_inputs(p_of, q_of, V, L, K, n, seed=11)
    res = oracle.verify_kseq(t, d, tok, 1.0, 21, 0, nthreads=8)
    keys = sorted(dist)
    index = {k: i for i, k in enumerate(keys)}
    counts = np.zeros(len(keys))
    for b in range(n):
        tau = int(res["accepted_len"][b])
        counts[index[tuple(int(v) for v in res["out_tokens"][b, :tau + 1])]] += 1
    expect = np.array([dist[k] for k in keys]) * n
    keep = expect > 5
    stat = ((counts[keep] - expect[keep]) ** 2 / expect[keep]).sum()
    assert stat < chi2.ppf(1 - 1e-6, int(keep.sum()) - 1), (stat, keep.sum())
    assert abs(res["accepted_len"].mean() - E_tau) < 5 * math.sqrt(L * L / n)


def test_eager_table_holds_what_the_procedure_uses():
    # rho_all[b, j, r] is solved for the number of drafts sharing draft j's first r tokens: at every position the
    # procedure visited, its rho is the eager entry of the retained draft of lowest index
    rng = np.random.default_rng(2)
    B, K, L, V = 60, 4, 3, 5
    t = rng.normal(0, 2, (B, 1, L + 1, V)).astype(np.float32).repeat(K, axis=1)       # rows shared, as in decoding
    d = rng.normal(0, 2, (B, 1, L, V)).astype(np.float32).repeat(K, axis=1)
    tok = rng.integers(0, 2, (B, K, L)).astype(np.int32)                              # many coinciding drafts
    res = oracle.verify_kseq(t, d, tok, 1.0, 0, 0, debug=True, eager=True)
    seen = 0
    for b in range(B):
        for r in range(L):
            if res["retained"][b, r] > 0:
                j = res["lead"][b, r]
                assert res["rho"][b, r] == res["rho_all"][b, j, r] and res["beta"][b, r] == res["beta_all"][b, j, r]
                same = sum(np.array_equal(tok[b, m, :r], tok[b, j, :r]) for m in range(K))
                assert res["retained"][b, r] == same
                seen += 1
    assert seen > B
