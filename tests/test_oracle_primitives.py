"""Pins for the building blocks of the CPU oracle (no GPU).

Each test checks one oracle function against something the paper or the
mathematics fixes, not against the oracle itself:
  * Philox4x32-10: the generator's published known-answer vectors + uniformity;
  * log-softmax: scipy's routine;
  * Eq. (hik) / Eq. (hLk) in the oracle's rescaled form: the literal equations
    evaluated in exact rational arithmetic, the hand-derived values of the golden
    file, and the K=1 reduction to greedy block verification (Section 3.3);
  * Eq. (pres): K=1 reduction norm(max{nu q - p, 0}) (Section 3.3);
  * inverse-CDF sampler: exact CDFs on tiny vocabularies.
"""
import itertools
import json
import math
import os
from fractions import Fraction as F

import numpy as np
import pytest
from scipy.special import log_softmax as scipy_log_softmax
from scipy.stats import chi2

import oracle
from oracle import exact_enum as ee

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- Philox

def test_philox_known_answers():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if ln[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        w = [int(v, 16) for v in r]
        assert oracle.philox4x32_10(w[0:4], w[4:6]) == tuple(w[6:10])


def test_uniform_is_word0_top_24_bits():
    seed, off, b, slot = 0x0123456789ABCDEF, 0xFEDCBA9876543210, 7, 13
    w = oracle.philox4x32_10([off & 0xFFFFFFFF, off >> 32, b, slot], [seed & 0xFFFFFFFF, seed >> 32])
    u = oracle.uniform(seed, off, b, slot)
    assert u == (w[0] >> 8) / 2 ** 24
    assert 0.0 <= u < 1.0
    assert float(np.float32(u)) == u          # exactly representable in float32


def test_uniform_slots_are_distinct_streams_and_uniform():
    n = 40000
    u = np.array([oracle.uniform(0, 0, b, s) for b in range(n // 8) for s in range(8)])
    counts, _ = np.histogram(u, bins=64, range=(0, 1))
    stat = ((counts - n / 64) ** 2 / (n / 64)).sum()
    assert stat < chi2.ppf(1 - 1e-6, 63)
    # neighbouring counters are uncorrelated
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03
    # offset and seed both change the stream
    assert oracle.uniform(0, 1, 0, 0) != oracle.uniform(0, 0, 0, 0)
    assert oracle.uniform(1, 0, 0, 0) != oracle.uniform(0, 0, 0, 0)


# ---------------------------------------------------------------- softmax

@pytest.mark.parametrize("T", [1.0, 0.4, 2.5])
def test_log_softmax_matches_scipy(T):
    rng = np.random.default_rng(1)
    z = rng.normal(0, 4, size=257)
    z[5] = 60.0
    z[9] = -300.0
    got, lse = oracle.log_softmax(z, T)
    np.testing.assert_allclose(got, scipy_log_softmax(z / T), rtol=0, atol=1e-12)
    assert abs(np.exp(got).sum() - 1) < 1e-12
    assert abs(lse - (z / T - got)[0]) < 1e-12


# ------------------------------------------------- Eq. (hik) / Eq. (hLk)

def _float_view(p_of, q_of, block, V):
    """(log nu, log P, log q row, log p row) of a block as floats from rational tables."""
    P, Q = ee.joint(p_of, block), ee.joint(q_of, block)
    lq = np.log([float(v) for v in q_of(block)])
    lp = np.log([float(v) for v in p_of(block)]) if True else None
    return math.log(Q) - math.log(P), math.log(P), lq, lp


@pytest.mark.parametrize("V,L,K", [(2, 2, 1), (2, 3, 2), (3, 2, 3), (3, 3, 4), (4, 2, 8), (2, 4, 16)])
def test_rescaled_h_equals_literal_equations(V, L, K):
    rng = np.random.default_rng(100 * V + 10 * L + K)
    for _ in range(3):
        p_of, q_of = ee.random_tables(rng, V, L)
        for r in range(1, L + 1):
            for block in itertools.product(range(V), repeat=r):
                exact = ee.h_literal(p_of, q_of, block, V, L, K)
                log_nu, log_P, lq, lp = _float_view(p_of, q_of, block, V)
                if r < L:
                    s = oracle.ot_sum(lq, lp, log_nu, K)
                    # the vocabulary sum itself, divided by q(x^i)
                    s_exact = ee.ot_sum_joint(p_of, q_of, block, V, K) / ee.joint(q_of, block)
                    assert abs(s - float(s_exact)) < 1e-13
                    got = oracle.h_sub(log_nu, log_P, s, K)
                else:
                    got = oracle.h_full(log_nu, log_P, K)
                assert abs(got - float(exact)) < 1e-11, (block, got, float(exact))
                assert 0.0 <= got <= 1.0


@pytest.mark.parametrize("V,L,K", [(2, 2, 1), (2, 3, 2), (3, 2, 3), (3, 3, 4), (4, 2, 8), (2, 4, 16), (5, 2, 5)])
def test_cancellation_free_h_equals_literal_equation_where_nu_exceeds_one(V, L, K):
    """Eq. (hik) for nu > 1 through the sum of non-negative terms (ot_excess, h_sub_excess) against the
    literal equation in exact rationals, and nu^2 (s - g) against the exact difference."""
    rng = np.random.default_rng(900 * V + 10 * L + K)
    seen = 0
    for _ in range(4):
        p_of, q_of = ee.random_tables(rng, V, L)
        for r in range(1, L):
            for block in itertools.product(range(V), repeat=r):
                P, Q = ee.joint(p_of, block), ee.joint(q_of, block)
                if Q <= P:
                    continue
                seen += 1
                exact = ee.h_literal(p_of, q_of, block, V, L, K)
                log_nu, log_P, lq, lp = _float_view(p_of, q_of, block, V)
                E = oracle.ot_excess(lq, lp, log_nu, K)
                nu = Q / P
                E_exact = nu * nu * (ee.ot_sum_joint(p_of, q_of, block, V, K) / Q - (1 - 1 / nu) ** K)
                assert E >= 0 and abs(E - float(E_exact)) <= 1e-11 * (1 + float(E_exact)), (block, E, float(E_exact))
                got = oracle.h_sub_excess(log_nu, log_P, E, K)
                assert abs(got - float(exact)) < 1e-11, (block, got, float(exact))
    assert seen >= 4


@pytest.mark.parametrize("K", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("eps_exp", [6, 12, 30, 120])
def test_cancellation_free_h_at_huge_block_ratios(K, eps_exp):
    """A drafted token of draft probability 10^-eps_exp gives its block a ratio nu of that order; the literal
    Eq. (hik), exact in rationals, has a finite value there, which the difference s - g cannot deliver in
    float64 (the plain form is checked to be off once nu exceeds 1e8: that is why the other form exists)."""
    eps = F(1, 10 ** eps_exp)
    # row 0: token 0 is nearly impossible under the draft, likely under the target
    p0 = [eps, F(2, 5) - eps, F(3, 5)]
    q0 = [F(1, 2), F(1, 4), F(1, 4)]
    # row 1 after token 0: an ordinary pair of distributions, one entry the target forbids almost entirely
    p1 = [F(1, 5), F(3, 10), F(1, 2)]
    q1 = [F(3, 10), F(3, 5), F(1, 10)]
    uni = [F(1, 3)] * 3
    def p_of(block): return p0 if block == () else (p1 if block == (0,) else uni)
    def q_of(block): return q0 if block == () else (q1 if block == (0,) else uni)
    V, L = 3, 3
    block = (0,)
    exact = ee.h_literal(p_of, q_of, block, V, L, K)
    assert 0 < exact <= 1
    log_nu = math.log(float(q0[0])) + eps_exp * math.log(10.0)
    log_P = -eps_exp * math.log(10.0)
    lq = np.log([float(v) for v in q1]); lp = np.log([float(v) for v in p1])
    got = oracle.h_sub_excess(log_nu, log_P, oracle.ot_excess(lq, lp, log_nu, K), K)
    assert abs(got - float(exact)) < 1e-11 * max(float(exact), 1e-3), (got, float(exact))
    if K >= 2 and eps_exp >= 12:
        plain = oracle.h_sub(log_nu, log_P, oracle.ot_sum(lq, lp, log_nu, K), K)
        assert abs(plain - float(exact)) > 1e-3, "the plain form is expected to have lost every digit here"


def test_cancellation_free_h_with_entries_of_zero_target_probability():
    # q[x] = 0 < p[x]: the entry adds nothing to s, but its draft mass enters through the linear term
    K = 3
    lq = np.array([math.log(0.6), math.log(0.4), -np.inf])
    lp = np.log([0.5, 0.3, 0.2])
    for nu in (1.5, 7.0, 1e9):
        log_nu = math.log(nu)
        q = np.array([0.6, 0.4, 0.0]); pp = np.array([0.5, 0.3, 0.2])
        t = np.maximum(1 - np.divide(pp, nu * q, out=np.full(3, np.inf), where=q > 0), 0)
        if nu < 1e4:
            s_minus_g = float((q * t ** K).sum() - (1 - 1 / nu) ** K)
            assert abs(oracle.ot_excess(lq, lp, log_nu, K) - nu * nu * s_minus_g) < 1e-9 * nu * nu
        # K a p t1^(K-1) from the masked entry alone is a lower bound
        assert oracle.ot_excess(lq, lp, log_nu, K) >= nu * K * 0.2 * (1 - 1 / nu) ** (K - 1) * (1 - 1e-12) - nu * nu * 0


def test_h_golden_hand_derived_values():
    doc = json.load(open(os.path.join(GOLDEN, "alg1_small_cases.json")))
    cases = {c["name"]: c for c in doc["cases"]}
    # values whose derivation is written out in the golden file's notes
    assert cases["CE1"]["K"]["2"]["h"] == {"0": "11/12", "1": "4/15"}
    assert cases["W2"]["K"]["2"]["h"]["0"] == "22/37"
    # the oracle reproduces every stored h of W2 from float logits
    half = lambda b: [F(1, 2), F(1, 2)]
    w2 = {(): [F(4, 5), F(1, 5)], (0,): [F(1, 4), F(3, 4)], (1,): [F(1, 2), F(1, 2)]}
    for a in range(2):
        for b in range(2):
            w2[(a, b)] = [F(1, 2), F(1, 2)]
    q_of = ee.table_from_dict(w2)
    for K in (1, 2, 3):
        for key, val in cases["W2"]["K"][str(K)]["h"].items():
            block = tuple(int(t) for t in key.split())
            log_nu, log_P, lq, lp = _float_view(half, q_of, block, 2)
            if len(block) < 2:
                got = oracle.h_sub(log_nu, log_P, oracle.ot_sum(lq, lp, log_nu, K), K)
            else:
                got = oracle.h_full(log_nu, log_P, K)
            assert abs(got - float(F(val))) < 1e-12, (K, key, got, val)


def _gbv_alpha(nu, q, p):
    """Acceptance probability of greedy block verification (Section 3.3), typed from its definition."""
    num = np.maximum(nu * q - p, 0).sum()
    den = np.maximum(p - nu * q, 0).sum()
    return num / den if den > 0 else 1.0


def test_K1_reduces_to_greedy_block_verification():
    rng = np.random.default_rng(7)
    V = 50
    for trial in range(40):
        q = rng.dirichlet(np.ones(V) * 0.3) + 1e-9
        q /= q.sum()
        p = rng.dirichlet(np.ones(V) * 0.3) + 1e-9
        p /= p.sum()
        nu = float(np.exp(rng.normal(0, 1.5)))
        log_P = float(-rng.uniform(0.1, 30))
        s = oracle.ot_sum(np.log(q), np.log(p), math.log(nu), 1)
        h = oracle.h_sub(math.log(nu), log_P, s, 1)
        assert abs(h - min(1.0, _gbv_alpha(nu, q, p))) < 1e-10
        # whole block: alpha(x^L) = nu_L, capped at one
        assert abs(oracle.h_full(math.log(nu), log_P, 1) - min(1.0, nu)) < 1e-12


def test_K1_L1_is_token_level_rejection():
    # Section 3.1: accept x with probability min{1, q(x)/p(x)}
    for qx, px in [(0.3, 0.5), (0.5, 0.3), (0.2, 0.2), (1e-9, 0.7)]:
        h = oracle.h_full(math.log(qx) - math.log(px), math.log(px), 1)
        assert abs(h - min(1.0, qx / px)) < 1e-12


def test_h_is_stable_for_tiny_block_probabilities():
    # joint probabilities far below double-precision resolution of 1 - (1-P)^K
    rng = np.random.default_rng(3)
    V, K = 64, 8
    q = rng.dirichlet(np.ones(V))
    p = rng.dirichlet(np.ones(V))
    log_nu = 0.7
    s = oracle.ot_sum(np.log(q), np.log(p), log_nu, K)
    ref = None
    for log_P in (-5.0, -40.0, -200.0, -700.0, -1200.0):
        h = oracle.h_sub(log_nu, log_P, s, K)
        assert 0 <= h <= 1
        if log_P <= -40:
            # c_K(P) -> K: h no longer depends on P
            nu = math.exp(log_nu)
            g = max(1 - 1 / nu, 0) ** K
            expect = nu * (s - g) / (K - nu * (1 - s))
            assert abs(h - expect) < 1e-12
            ref = h
    assert ref is not None


def test_h_denominator_zero_reads_as_one():
    # p == q and nu == 1 at K == 1: numerator and denominator of Eq. (hik) both vanish
    q = np.array([0.25, 0.75])
    s = oracle.ot_sum(np.log(q), np.log(q), 0.0, 1)
    assert s == 0.0
    assert oracle.h_sub(0.0, math.log(1.0), s, 1) == 1.0


# ------------------------------------------------------------- Eq. (pres)

def test_residual_K1_is_gbv_residual():
    rng = np.random.default_rng(11)
    V = 40
    q = rng.dirichlet(np.ones(V))
    p = rng.dirichlet(np.ones(V))
    for nu in (0.3, 1.0, 2.2):
        w = np.array([oracle.ot_sum(np.log(q[x:x + 1]), np.log(p[x:x + 1]), math.log(nu), 1) for x in range(V)])
        ref = np.maximum(nu * q - p, 0)          # Section 3.3 residual, up to normalisation
        np.testing.assert_allclose(w / w.sum(), ref / ref.sum(), atol=1e-14)


def test_residual_matches_literal_equation():
    rng = np.random.default_rng(5)
    V, L, K = 3, 2, 3
    p_of, q_of = ee.random_tables(rng, V, L)
    for block in [(), (0,), (2,)]:
        exact, deg = ee.residual_literal(p_of, q_of, block, V, K)
        log_nu, _, lq, lp = _float_view(p_of, q_of, block, V)
        w = np.array([oracle.ot_sum(lq[x:x + 1], lp[x:x + 1], log_nu, K) for x in range(V)])
        if not deg:
            np.testing.assert_allclose(w / w.sum(), [float(v) for v in exact], atol=1e-13)


# ------------------------------------------------------- inverse-CDF draw

def test_sample_cdf_exact_intervals():
    w = np.array([0.0, 2.0, 0.0, 1.0, 5.0, 0.0])
    W = 8.0
    edges = [(0.0, 1), (0.2499, 1), (0.25, 3), (0.3749, 3), (0.375, 4), (0.999999, 4)]
    for u, y in edges:
        got, tot, margin = oracle.sample_cdf(w, u)
        assert (got, tot) == (y, W)
    # strict inequality: u*W equal to a running sum moves on to the next positive token
    assert oracle.sample_cdf(w, 0.25)[0] == 3
    # margin = distance to the nearer interval end, relative to W
    y, _, margin = oracle.sample_cdf(w, 0.30)
    assert y == 3 and abs(margin - 0.05) < 1e-15
    # all-zero weights are reported, not sampled
    assert oracle.sample_cdf(np.zeros(4), 0.5)[0] == -1


def test_sample_cdf_law():
    w = np.array([3.0, 1.0, 0.0, 4.0])
    n = 1 << 12
    ys = [oracle.sample_cdf(w, (j + 0.5) / n)[0] for j in range(n)]
    counts = np.bincount(ys, minlength=4)
    np.testing.assert_array_equal(counts, (w / w.sum() * n).astype(int))
