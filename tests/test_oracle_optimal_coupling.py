"""The single-position optimal coupling (oracle/optimal_coupling.py): what any distribution-preserving multi-draft
verifier can accept at most, set against the closed form of Theorem 5.3, Algorithm 1 as printed and the K-SEQ rule
of Section 3.2.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import exact_enum as ee
from oracle import optimal_coupling as oc


def _tables(seed, n):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        V = int(rng.integers(2, 5))
        K = int(rng.integers(1, 4))
        p = rng.dirichlet(np.ones(V) * rng.uniform(0.3, 2.0))
        q = rng.dirichlet(np.ones(V) * rng.uniform(0.3, 2.0))
        yield V, K, p, q


def test_one_draft_is_the_overlap_of_the_two_models():
    # K = 1: the maximal coupling of p and q, P(X = Y) = sum_x min{p, q} (textbook)
    for V, _, p, q in _tables(1, 40):
        assert oc.optimal_acceptance(p, q, 1) == pytest.approx(float(np.minimum(p, q).sum()), abs=1e-9)


def test_hand_values():
    p, q = [Fraction(1, 2)] * 2, [Fraction(4, 5), Fraction(1, 5)]
    # K = 2: the three tuples containing token 0 (mass 3/4) can all emit 0, and q(1) = 1/5 fits into the tuples
    # containing 1, so 3/4 + 1/5; K = 3: only (1,1,1) lacks 0 and only (0,0,0) lacks 1, each of mass 1/8 <= q
    assert oc.optimal_acceptance(p, q, 2) == pytest.approx(0.95, abs=1e-9)
    assert oc.optimal_acceptance(p, q, 3) == pytest.approx(1.0, abs=1e-9)
    assert oc.optimal_acceptance(q, q, 2) == pytest.approx(1.0, abs=1e-9)        # identical models: always accept


def test_linear_program_equals_min_cut():
    for V, K, p, q in _tables(2, 120):
        assert oc.optimal_acceptance(p, q, K) == pytest.approx(oc.optimal_acceptance_min_cut(p, q, K), abs=1e-9)


def test_more_drafts_never_hurt_the_optimum():
    for V, _, p, q in _tables(3, 30):
        a = [oc.optimal_acceptance_min_cut(p, q, K) for K in (1, 2, 3, 4)]
        assert all(a[i] <= a[i + 1] + 1e-12 for i in range(3))


def test_order_of_the_four_figures():
    """optimum >= closed form of Theorem 5.3 >= ... and optimum >= K-SEQ (a valid rule); the printed Algorithm 1
    stays below the closed form for K >= 2 and its output is not q there (reading R11)."""
    cases = [([Fraction(1, 2)] * 2, [Fraction(4, 5), Fraction(1, 5)]),
             ([Fraction(1, 2), Fraction(1, 3), Fraction(1, 6)], [Fraction(1, 6), Fraction(1, 3), Fraction(1, 2)])]
    for p, q in cases:
        for K, opt, cf, alg, tv, ks in oc.single_position_table(p, q, Ks=(1, 2, 3)):
            assert opt >= cf - 1e-9 and opt >= ks - 1e-9
            if K == 1:
                assert opt == pytest.approx(cf, abs=1e-9) and alg == pytest.approx(cf, abs=1e-12)
                assert ks == pytest.approx(cf, abs=1e-9) and tv == 0.0
            else:
                assert alg < cf - 1e-3 and tv > 1e-3


def test_closed_form_never_exceeds_the_optimum():
    for V, K, p, q in _tables(4, 200):
        assert oc.closed_form_single_position(p, q, K) <= oc.optimal_acceptance_min_cut(p, q, K) + 1e-12


def test_closed_form_matches_the_enumerations_value():
    p = [Fraction(1, 2), Fraction(1, 3), Fraction(1, 6)]
    q = [Fraction(1, 6), Fraction(1, 3), Fraction(1, 2)]
    for K in (1, 2, 3):
        want = ee.closed_form_E_tau(lambda b: p, lambda b: q, 3, 1, K)
        assert oc.closed_form_single_position(p, q, K) == pytest.approx(float(want), abs=1e-12)
