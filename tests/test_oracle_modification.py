"""Pins of the oracle's distribution modification (Algorithm 2) -- CPU only.

The oracle evaluates Algorithm 2 in the rescaled per-token form (block ratio carried in logs);
these tests pin it to the printed expression in exact rationals, to the single-draft form of
greedy block verification (Section 3.3), and to Theorem 4.2's statement about the complete
output O = (t^tau, y, x^(L-tau-1)).
"""
import itertools
from fractions import Fraction as F

import numpy as np
import pytest

import oracle
from oracle import exact_enum as ee
from specgbv_synth import tables_to_inputs


def _rows_for_prefix(p_of, q_of, prefix, tokens, V):
    """Logit rows (float32 logs of the table probabilities) conditioned on prefix + tokens[:r]."""
    M = len(tokens)
    t = np.empty((1, 1, M, V), np.float32)
    d = np.empty((1, 1, M, V), np.float32)
    for r in range(M):
        blk = tuple(prefix) + tuple(tokens[:r])
        t[0, 0, r] = np.log([float(v) for v in q_of(blk)])
        d[0, 0, r] = np.log([float(v) for v in p_of(blk)])
    return t, d


@pytest.mark.parametrize("V,L", [(2, 2), (2, 3), (3, 2), (3, 3)])
def test_theorem_4_2_complete_output_is_target_at_k1(V, L):
    rng = np.random.default_rng(10 * V + L)
    p_of, q_of = ee.random_tables(rng, V, L)
    full = ee.enumerate_full_output(p_of, q_of, V, L, 1)
    for blk in itertools.product(range(V), repeat=L):
        assert full.get(blk, F(0)) == ee.joint(q_of, blk)            # exactly q(x^L)


def test_complete_output_for_k2_is_not_the_target():
    # the printed Algorithm 1 is not distribution preserving for K >= 2; Algorithm 2 does not repair it
    rng = np.random.default_rng(3)
    p_of, q_of = ee.random_tables(rng, 2, 3)
    full = ee.enumerate_full_output(p_of, q_of, 2, 3, 2)
    tv = sum(abs(full.get(b, F(0)) - ee.joint(q_of, b)) for b in itertools.product(range(2), repeat=3)) / 2
    assert tv > F(1, 100)


@pytest.mark.parametrize("K", [1, 2, 3, 5])
def test_modify_values(K):
    """Row by row against exact rationals: K drafts share the carried ratio, each continues it
    along its own tokens with the original target probabilities."""
    rng = np.random.default_rng(50 + K)
    V, depth = 3, 4
    p_of, q_of = ee.random_tables(rng, V, depth)
    prefixes = list(itertools.product(range(V), repeat=1)) + list(itertools.product(range(V), repeat=2))
    for prefix in prefixes:
        M = 2
        tok = rng.integers(0, V, (K, M)).astype(np.int32)
        t = np.empty((1, K, M, V), np.float32)
        d = np.empty((1, K, M, V), np.float32)
        for k in range(K):
            tk, dk = _rows_for_prefix(p_of, q_of, prefix, tuple(int(v) for v in tok[k]), V)
            t[0, k], d[0, k] = tk[0, 0], dk[0, 0]
        carry = float(np.log(float(ee.joint(q_of, prefix) / ee.joint(p_of, prefix))))
        res = oracle.modify(t, d, tok.reshape(1, K, M), 1.0, [carry], [M])
        for k in range(K):
            for r in range(M):
                blk = tuple(prefix) + tuple(int(v) for v in tok[k, :r])
                want, deg = ee.modified_literal(p_of, q_of, blk, V, K)
                got = np.exp(res["logq"][0, k, r])
                assert int(res["fallback"][0, k, r]) == int(deg)
                # tables pass through float32 logits: 1e-6 is their rounding, far below any formula error
                np.testing.assert_allclose(got, [float(v) for v in want], rtol=0, atol=2e-6)
                assert abs(got.sum() - 1.0) < 1e-12


def test_k1_modification_is_greedy_block_verification():
    # Section 3.3: the single-draft modification is norm(max{nu q - p, 0})
    rng = np.random.default_rng(7)
    V, M = 40, 3
    t = rng.normal(0, 2, (2, 1, M, V)).astype(np.float32)
    d = (t + rng.normal(0, 1, (2, 1, M, V))).astype(np.float32)
    tok = rng.integers(0, V, (2, 1, M)).astype(np.int32)
    carry = np.array([0.3, -0.8])
    T = float(np.float32(0.9))                           # the entry point takes a float32 temperature
    res = oracle.modify(t, d, tok, T, carry, [M, 1])
    for b in range(2):
        lognu = carry[b]
        for r in range(M):
            lq, _ = oracle.log_softmax(t[b, 0, r], T)
            lp, _ = oracle.log_softmax(d[b, 0, r], T)
            if r < (M, 1)[b]:
                w = np.maximum(np.exp(lognu) * np.exp(lq) - np.exp(lp), 0.0)
                want = w / w.sum()
            else:
                want = np.exp(lq)
            np.testing.assert_allclose(np.exp(res["logq"][b, 0, r]), want, rtol=1e-9, atol=1e-12)   # nu q - p cancels near zero
            lognu += lq[tok[b, 0, r]] - lp[tok[b, 0, r]]


def test_all_zero_weights_leave_the_row_unchanged():
    # p == q and nu = 1: every weight vanishes; the row stays q (same reading as for the residual)
    z = np.log(np.array([[[[0.2, 0.3, 0.5]]]], np.float32))
    res = oracle.modify(z, z.copy(), np.zeros((1, 1, 1), np.int32), 1.0, [0.0], [1])
    assert res["fallback"][0, 0, 0] == 1 and res["norm"][0, 0, 0] == 1.0
    np.testing.assert_allclose(np.exp(res["logq"][0, 0, 0]), [0.2, 0.3, 0.5], rtol=1e-6)


def test_verify_reports_the_carried_ratio_and_count():
    rng = np.random.default_rng(11)
    V, L, K, n = 3, 3, 2, 400
    p_of, q_of = ee.random_tables(rng, V, L)
    target, draft, tokens = tables_to_inputs(p_of, q_of, V, L, K, n, seed=5)
    res = oracle.verify(target, draft, tokens, 1.0, 3, 0, debug=True)
    for b in range(n):
        tau = int(res["accepted_len"][b])
        out = tuple(int(v) for v in res["out_tokens"][b, :tau + 1])
        if tau == L:
            assert res["modify_count"][b] == 0
            continue
        assert res["modify_count"][b] == L - tau - 1
        want = float(np.log(float(ee.joint(q_of, out) / ee.joint(p_of, out))))
        assert abs(res["carry_log_nu"][b] - want) < 1e-5               # tables pass through float32 logits


# ------------------------------------------------ several iterations (Algorithm 3)

def _prefix_law(text_law, m):
    law = {}
    for text, pr in text_law.items():
        law[text[:m]] = law.get(text[:m], F(0)) + pr
    return law


@pytest.mark.parametrize("V,L,iters", [(2, 2, 3), (2, 3, 3), (3, 3, 2)])
def test_decoded_text_is_target_distributed_over_several_iterations_at_k1(V, L, iters):
    """Algorithm 3 with q updated in place (pending modifications stay in force and compose):
    the first `iters` decoded tokens follow the target model exactly."""
    rng = np.random.default_rng(40 + 10 * V + L)
    p2, q2 = ee.random_tables(rng, V, 2)
    p_of = lambda b: p2(tuple(b[-2:]))
    q_of = lambda b: q2(tuple(b[-2:]))
    law = _prefix_law(ee.enumerate_decoding(p_of, q_of, V, L, 1, iters), iters)
    for blk in itertools.product(range(V), repeat=iters):
        assert law.get(blk, F(0)) == ee.joint(q_of, blk)


def test_forgetting_a_pending_modification_changes_the_law():
    # L = 3: after tau = 0 two rows are modified; if the next iteration emits one token, the second
    # modified row must survive into the third iteration.  Laying each modification over the
    # original q instead is not distribution preserving.
    rng = np.random.default_rng(62)
    p2, q2 = ee.random_tables(rng, 2, 2)
    p_of = lambda b: p2(tuple(b[-2:]))
    q_of = lambda b: q2(tuple(b[-2:]))
    law = _prefix_law(ee.enumerate_decoding(p_of, q_of, 2, 3, 1, 3, compose=False), 3)
    tv = sum(abs(law.get(b, F(0)) - ee.joint(q_of, b)) for b in itertools.product(range(2), repeat=3)) / 2
    assert tv > F(1, 1000)
    # with L = 2 a modification never outlives the next iteration: both readings coincide
    a = ee.enumerate_decoding(p_of, q_of, 2, 2, 1, 3, compose=False)
    b = ee.enumerate_decoding(p_of, q_of, 2, 2, 1, 3, compose=True)
    assert a == b


def test_carry_advance_follows_the_joint_ratio():
    """The pending block ratio after an iteration is the joint ratio q/p of everything emitted since
    the modification was made, under the rows that modification modifies."""
    rng = np.random.default_rng(17)
    V, L, K, n = 3, 4, 2, 300
    p_of, q_of = ee.random_tables(rng, V, L + 1)
    target, draft, tokens = tables_to_inputs(p_of, q_of, V, L, K, n, seed=9)
    res = oracle.verify(target, draft, tokens, 1.0, 21, 0, debug=True)
    carry0 = rng.normal(0, 0.3, n)
    count0 = rng.integers(0, L, n).astype(np.int32)
    carry, count = oracle.carry_advance(target, draft, tokens, res["accepted_len"], res["accepted_draft_idx"],
                                        res["out_tokens"], 1.0, carry0, count0)
    seen = 0
    for b in range(n):
        tau = int(res["accepted_len"][b])
        if tau == L or count0[b] <= tau + 1:
            assert count[b] == 0
            continue
        seen += 1
        emitted = tuple(int(v) for v in res["out_tokens"][b, :tau + 1])
        want = carry0[b] + float(np.log(float(ee.joint(q_of, emitted) / ee.joint(p_of, emitted))))
        assert count[b] == count0[b] - (tau + 1)
        assert abs(carry[b] - want) < 1e-5                  # tables pass through float32 logits
    assert seen > 10
