"""The GPU path's output law against the exact law of Algorithm 1 (needs an MI355X: -m gpu).

Parity with the oracle is checked call by call elsewhere; this test looks at the GPU path alone:
over many independent prefixes that share small conditional tables, the frequencies of the
outputs (t^tau, y) produced by libspecgbv.so must match the law obtained by enumerating every
draft tuple and every accept/reject branch of Algorithm 1 in exact rationals.  For K = 1 that
law is the target distribution itself (Theorem 4.2); for K >= 2 it is the law of the printed
algorithm (which is not the target distribution: already for two tokens, one position and two
drafts the exact enumeration gives 5/36 where the target has 1/5 -- case CE1 of
tests/golden/alg1_small_cases.json).
"""
from fractions import Fraction as F

import numpy as np
import pytest
from scipy.stats import chi2

from oracle import exact_enum as ee
from parity_util import run_gpu
from specgbv_synth import tables_to_inputs

pytestmark = pytest.mark.gpu

# Section 4.2-style worked example (V = 2, L = 2): p uniform, q(.|()) = (4/5, 1/5),
# q(.|0) = (1/4, 3/4), q(.|1) = (1/2, 1/2)
W2 = {(): [F(4, 5), F(1, 5)], (0,): [F(1, 4), F(3, 4)], (1,): [F(1, 2), F(1, 2)]}
for _a in range(2):
    for _b in range(2):
        W2[(_a, _b)] = [F(1, 2), F(1, 2)]


def _gpu_counts(p_of, q_of, V, L, K, n, seed):
    counts, tau_sum = {}, 0
    chunk = 50_000
    for c, start in enumerate(range(0, n, chunk)):
        m = min(chunk, n - start)
        target, draft, tokens = tables_to_inputs(p_of, q_of, V, L, K, m, seed + c)
        res = run_gpu(target, draft, tokens, 1.0, 17, c, algo="auto")
        out, tau, f = res["out_tokens"], res["accepted_len"], res["accepted_draft_idx"]
        assert np.all((f == -1) == (tau == 0))
        for j in range(L + 1):
            assert np.all((out[:, j] == -1) == (j > tau))
        idx = np.nonzero(tau > 0)[0]
        for j in range(L):
            sel = idx[tau[idx] > j]
            assert np.array_equal(out[sel, j], tokens[sel, f[sel], j])     # accepted tokens are the draft's
        keys, cnt = np.unique(out, axis=0, return_counts=True)
        for krow, cc in zip(keys, cnt):
            key = tuple(int(t) for t in krow if t >= 0)
            counts[key] = counts.get(key, 0) + int(cc)
        tau_sum += int(tau.sum())
    return counts, tau_sum / n


@pytest.mark.parametrize("K,n", [(1, 400_000), (2, 200_000), (3, 200_000)])
def test_gpu_law_on_worked_example(K, n):
    half = lambda b: [F(1, 2), F(1, 2)]
    q_of = lambda b: W2[tuple(b)]
    dist, E_tau, _ = ee.enumerate_alg1(half, q_of, 2, 2, K)
    counts, tau_mean = _gpu_counts(half, q_of, 2, 2, K, n, seed=100 + K)
    assert set(counts) <= {k for k, v in dist.items() if v > 0}, "outcome outside the exact support"
    stat, dof = 0.0, -1
    for key, pr in dist.items():
        e = float(pr) * n
        if e == 0:
            continue
        stat += (counts.get(key, 0) - e) ** 2 / e
        dof += 1
    assert stat < chi2.ppf(1 - 1e-6, dof), "chi-squared %.1f on %d degrees of freedom" % (stat, dof)
    assert abs(tau_mean - float(E_tau)) < 6.0 * 2.0 / np.sqrt(n)           # |tau| <= L = 2
    if K == 1:
        # Theorem 4.2: the first output token is distributed as q(.|prefix) = (4/5, 1/5)
        first0 = sum(c for k, c in counts.items() if k[0] == 0) / n
        assert abs(first0 - 0.8) < 6.0 * np.sqrt(0.8 * 0.2 / n)


def test_gpu_law_random_tables_three_tokens():
    rng = np.random.default_rng(5)
    V, L, K = 3, 2, 2
    p_of, q_of = ee.random_tables(rng, V, L)
    dist, E_tau, _ = ee.enumerate_alg1(p_of, q_of, V, L, K)
    n = 200_000
    counts, tau_mean = _gpu_counts(p_of, q_of, V, L, K, n, seed=7)
    stat, dof = 0.0, -1
    for key, pr in dist.items():
        e = float(pr) * n
        if e == 0:
            assert counts.get(key, 0) == 0
            continue
        stat += (counts.get(key, 0) - e) ** 2 / e
        dof += 1
    assert stat < chi2.ppf(1 - 1e-6, dof), "chi-squared %.1f on %d degrees of freedom" % (stat, dof)
    assert abs(tau_mean - float(E_tau)) < 6.0 * 2.0 / np.sqrt(n)
