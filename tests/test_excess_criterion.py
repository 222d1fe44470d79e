"""The rule by which the kernels decide that a row's plain Eq. (hik) sum is good enough, checked on the CPU against
the oracle's two forms of the acceptance probability.

For a block ratio nu > 1 the kernels have s = sum_x q max(1 - p/(nu q), 0)^K from a float32 sweep (relative error up to
2e-7 + 1.3e-7 K on rows that a few entries dominate) and g = (1 - 1/nu)^K; Eq. (hik) needs nu (s - g).  They take the sum
again as E = nu^2 (s - g), term by term and without the difference, only where two tests say so (written out below as
the kernels have them: `excess_wanted`, then `excess_needed`).  The property that makes the rule sound: wherever it
says "the plain sum will do", the oracle's plain form of h evaluated at s (1 +- eps_s(K)) stays within the bar the
acceptance probability is held to, 1e-5 |h| + 1e-9, of the oracle's cancellation-free form at the exact E.  Sweeps
over nu, P, K and the size of s - g, including the corners (s - g far below the error of s, Q = nu P near one,
K = 1).  No GPU involved: this pins the rule, the GPU parity tests pin its implementation."""
import math

import numpy as np
import pytest

import oracle

def eps_s(K):
    """Relative error allowed for on the float32 sum: 3e-7 observed at K = 4, 1.3e-6 at K = 9 on a row that one entry dominates."""
    return 2.0e-7 + 1.3e-7 * K


def cancel_factor(K):
    """Largest s / (s - g) the plain sum serves up to: times eps_s(K) it is half the bar (float32 in the kernels)."""
    return min(16.0, 38.5 / (1.54 + K))


def plain_sum_suffices(log2nu, log2P, s, K):
    """The kernels' rule (same operations, float64 here where the first test runs in float32)."""
    if not log2nu > 0.0:
        return True                                   # nu <= 1: Eq. (hik) has no difference
    inv_nu = 2.0 ** -log2nu
    t1 = 1.0 - inv_nu
    g = t1 ** K
    f = cancel_factor(K)
    if not (s - g) * f < s:                           # first test: the difference keeps enough bits of s
        return True
    if K == 1:
        return True                                   # h = 1 whatever E is
    P = 2.0 ** log2P
    U, S2, pw = 1.0, 0.0, 1.0
    for _ in range(1, K):
        S2 += U
        pw *= t1
        U = (1.0 - P) * U + pw
    one_Q = max(1.0 - 2.0 ** (log2nu + log2P), 0.0)
    D = inv_nu * one_Q * S2
    x = (s - g) - (16.0e-6 / f) * s                   # low end of what the plain s allows for s - g
    if not x > 0.0:
        return False
    return not x * f * (D + x / inv_nu) < s * D


def _cases(seed, n):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        K = int(rng.choice([1, 2, 3, 4, 8, 16]))
        log2nu = float(2.0 ** rng.uniform(-8, 7.5))                  # nu from 1.003 to 2^180
        nu = 2.0 ** log2nu
        # Q = nu P <= 1: from nearly one down to tiny
        log2Q = -float(2.0 ** rng.uniform(-20, 6))
        log2P = log2Q - log2nu
        g = (1.0 - 1.0 / nu) ** K
        # s - g relative to what is left above g, over many orders of magnitude
        room = 1.0 - g
        x = room * float(10.0 ** rng.uniform(-14, 0)) if room > 0 else 0.0
        yield K, log2nu, log2P, g, x


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_where_the_rule_keeps_the_plain_sum_the_plain_form_is_within_the_bar(seed):
    kept = taken = 0
    ln2 = math.log(2.0)
    for K, log2nu, log2P, g, x in _cases(seed, 4000):
        s = g + x
        if s - g <= 0.0:
            continue                                                 # x lost in float64: not representable as a case
        x = s - g                                                    # what float64 kept of it
        nu = 2.0 ** log2nu
        h_true = oracle.h_sub_excess(log2nu * ln2, log2P * ln2, nu * nu * x, K)
        for d in (-eps_s(K), eps_s(K)):
            s_seen = s * (1.0 + d)
            if plain_sum_suffices(log2nu, log2P, s_seen, K):
                kept += 1
                h_plain = oracle.h_sub(log2nu * ln2, log2P * ln2, s_seen, K)
                assert abs(h_plain - h_true) <= 1.0e-5 * abs(h_true) + 1.0e-9, (K, log2nu, log2P, g, x, d, h_plain, h_true)
            else:
                taken += 1
    assert kept > 1000 and taken > 1000, (kept, taken)               # the sweep reaches both sides of the rule


def test_corners():
    # s - g far below the error of s: always taken again
    assert not plain_sum_suffices(140.0, -150.0, 1.0 - 1e-9, 8)
    # K = 1, nu > 1: h = 1, never taken
    assert plain_sum_suffices(3.0, -5.0, (1 - 2.0 ** -3) * (1 + 1e-9), 1)
    # a block accepted almost surely (Q = nu P = 1 - 1e-12: D vanishes) does not care about s - g
    assert plain_sum_suffices(2.0, math.log2(1 - 1e-12) - 2.0, 0.75 ** 4 * (1 + 1e-3), 4)
    # nu <= 1: no difference in Eq. (hik)
    assert plain_sum_suffices(-1.0, -3.0, 0.2, 4)
