"""Exact-rational brute force of SpecTr-GBV on tiny vocabularies.

TEST INFRASTRUCTURE ONLY (like the rest of oracle/).  Independent of
specgbv_oracle.c: it evaluates the paper's equations *literally* (with the
joint block probabilities p(x^i), q(x^i) of Eq. (hik), Eq. (hLk), Eq. (pres)) in
``fractions.Fraction`` and enumerates every K-tuple of drafts and every
accept/reject branch of Algorithm 1.  The C oracle's rescaled formulas, its scan
and its Monte-Carlo behaviour are pinned against these exact values.
"""
from __future__ import annotations

import itertools
from fractions import Fraction
from typing import Callable, Dict, Tuple

Block = Tuple[int, ...]
Table = Callable[[Block], list]


def joint(table: Table, block: Block) -> Fraction:
    """Probability of a token block under an autoregressive table."""
    pr = Fraction(1)
    for j, t in enumerate(block):
        pr *= table(block[:j])[t]
    return pr


def _one_minus_min_pow(pb: Fraction, qb: Fraction, K: int) -> Fraction:
    """(1 - min{p/q, 1})^K; a block the target gives probability 0 has min{p/q, 1} = 1."""
    if qb == 0:
        return Fraction(0)
    ratio = pb / qb
    return (1 - min(ratio, Fraction(1))) ** K


def ot_sum_joint(p_of: Table, q_of: Table, block: Block, V: int, K: int) -> Fraction:
    """sum_x q(x^i, x) (1 - min{p(x^i,x)/q(x^i,x), 1})^K  -- the vocabulary sum of Eq. (hik)."""
    tot = Fraction(0)
    for x in range(V):
        ext = block + (x,)
        tot += joint(q_of, ext) * _one_minus_min_pow(joint(p_of, ext), joint(q_of, ext), K)
    return tot


def h_literal(p_of: Table, q_of: Table, block: Block, V: int, L: int, K: int) -> Fraction:
    """Acceptance probability of a block: Eq. (hik) for len < L, Eq. (hLk) for len = L."""
    P, Q = joint(p_of, block), joint(q_of, block)
    if len(block) == L:
        return Q * (1 - _one_minus_min_pow(P, Q, K)) / (1 - (1 - P) ** K)
    S = ot_sum_joint(p_of, q_of, block, V, K)
    num = S - Q * _one_minus_min_pow(P, Q, K)
    den = 1 - (1 - P) ** K - Q + S
    if den == 0:
        return Fraction(1)          # 0/0 read as its limit
    h = num / den
    assert 0 <= h <= 1, (block, h)
    return h


def residual_literal(p_of: Table, q_of: Table, block: Block, V: int, K: int):
    """Eq. (pres): distribution of the token after the accepted block (length < L).

    Returns (distribution, degenerate) where degenerate marks the all-zero case, read as
    a draw from q(.|block)."""
    w = []
    for x in range(V):
        ext = block + (x,)
        w.append(joint(q_of, ext) * _one_minus_min_pow(joint(p_of, ext), joint(q_of, ext), K))
    tot = sum(w)
    if tot == 0:
        return list(q_of(block)), True
    return [v / tot for v in w], False


def closed_form_E_tau(p_of: Table, q_of: Table, V: int, L: int, K: int) -> Fraction:
    """Right-hand side of Lemma 5.1 / Theorem 5.3."""
    tot = Fraction(0)
    for t in range(1, L + 1):
        for block in itertools.product(range(V), repeat=t):
            P, Q = joint(p_of, block), joint(q_of, block)
            tot += Q * (1 - _one_minus_min_pow(P, Q, K))
    return tot


def _scan_branches(drafts, hval, K: int, L: int):
    """All (probability, tau, f) leaves of Algorithm 1's loop for fixed drafts."""
    leaves = []

    def rec(k, i, start_done, tau, f, H, pr):
        # (k, i): next test is sub-block length i of draft k; i runs tau_at_entry+1 .. L
        if pr == 0:
            return
        if k == K:
            leaves.append((pr, tau, f))
            return
        if i > L:
            rec(k + 1, tau + 1, False, tau, f, H, pr)
            return
        block = drafts[k][:i]
        if block in H:
            rec(k, i + 1, True, tau, f, H, pr)
            return
        h = hval(block)
        # accept
        if i == L:
            leaves.append((pr * h, L, k))            # break
        else:
            rec(k, i + 1, True, i, k, H, pr * h)
        # reject
        rec(k, i + 1, True, tau, f, H | {block}, pr * (1 - h))

    rec(0, 1, False, 0, -1, frozenset(), Fraction(1))
    return leaves


def enumerate_alg1(p_of: Table, q_of: Table, V: int, L: int, K: int):
    """Exact law of Algorithm 1's output.

    Returns (dist, E_tau, degenerate_mass): dist maps the output token tuple
    (t^tau followed by y) to its probability.
    """
    hcache: Dict[Block, Fraction] = {}

    def hval(block):
        if block not in hcache:
            hcache[block] = h_literal(p_of, q_of, block, V, L, K)
        return hcache[block]

    rcache = {}
    dist: Dict[Block, Fraction] = {}
    E_tau = Fraction(0)
    degenerate_mass = Fraction(0)
    blocks = list(itertools.product(range(V), repeat=L))
    for drafts in itertools.product(blocks, repeat=K):
        pd = Fraction(1)
        for d in drafts:
            pd *= joint(p_of, d)
        if pd == 0:
            continue
        for pr, tau, f in _scan_branches(drafts, hval, K, L):
            w = pd * pr
            if w == 0:
                continue
            E_tau += w * tau
            t = drafts[f][:tau] if tau > 0 else ()
            if tau == L:
                ydist, deg = list(q_of(t)), False
            else:
                if t not in rcache:
                    rcache[t] = residual_literal(p_of, q_of, t, V, K)
                ydist, deg = rcache[t]
            if deg:
                degenerate_mass += w
            for y in range(V):
                if ydist[y] != 0:
                    key = t + (y,)
                    dist[key] = dist.get(key, Fraction(0)) + w * ydist[y]
    assert sum(dist.values()) == 1
    return dist, E_tau, degenerate_mass


def modified_literal(p_of: Table, q_of: Table, prefix: Block, V: int, K: int):
    """Algorithm 2: q_new(. | prefix) for prefix = (t^tau, y, x^(i-1)), written with the joint
    probabilities of the whole sequence exactly as printed.  It is the expression of Eq. (pres)
    evaluated at that longer block; all-zero weights are read as q(. | prefix)."""
    return residual_literal(p_of, q_of, prefix, V, K)


def enumerate_full_output(p_of: Table, q_of: Table, V: int, L: int, K: int):
    """Exact law of the first L tokens of O = (t^tau, y, x^(L-tau-1)) of Theorem 4.2: Algorithm 1's
    output completed with tokens drawn one by one from Algorithm 2's modified distributions."""
    dist, _, _ = enumerate_alg1(p_of, q_of, V, L, K)
    out: Dict[Block, Fraction] = {}

    def extend(prefix, pr):
        if pr == 0:
            return
        if len(prefix) >= L:
            key = prefix[:L]
            out[key] = out.get(key, Fraction(0)) + pr
            return
        qn, _ = modified_literal(p_of, q_of, prefix, V, K)
        for x in range(V):
            extend(prefix + (x,), pr * qn[x])

    for key, pr in dist.items():
        extend(key, pr)
    assert sum(out.values()) == 1
    return out


def enumerate_decoding(p_of: Table, q_of: Table, V: int, L: int, K: int, iters: int, compose: bool = True):
    """Exact law of the text decoded by `iters` iterations of Algorithm 3 (draft, verify with
    Algorithm 1, update q with Algorithm 2), as {token tuple: probability}.

    Algorithm 3 updates q in place, so the target of an iteration is the q left by all earlier
    modifications, and Algorithm 2 is evaluated with that q: a modification whose rows are not
    used up when the next iteration ends is thereby carried into the next one.
    compose=False is the reading that does NOT do this: the block ratio of (t^tau, y) is taken
    from the iteration as it was verified, but the rows being modified, and the continuation of
    the ratio along them, are the ORIGINAL q.  It exists to show that the readings differ."""
    out: Dict[Block, Fraction] = {}

    def run(prefix: Block, pr: Fraction, target_of: Table, it: int):
        if it == iters:
            out[prefix] = out.get(prefix, Fraction(0)) + pr
            return
        n0 = len(prefix)
        p_rel = lambda b: p_of(prefix + tuple(b))
        q_rel = lambda b: target_of(prefix + tuple(b))
        dist, _, _ = enumerate_alg1(p_rel, q_rel, V, L, K)
        for key, w in dist.items():
            tau = len(key) - 1
            count = L - tau - 1 if tau < L else 0
            new_prefix = prefix + key
            memo: Dict[Block, list] = {}

            def new_target(block, _np=new_prefix, _count=count, _memo=memo, _key=key):
                block = tuple(block)
                j = len(block) - len(_np)
                if not (0 <= j < _count and block[:len(_np)] == _np):
                    return target_of(block) if compose else q_of(block)
                if block not in _memo:
                    if compose:
                        # Algorithm 2 as printed: joint probabilities of (t^tau, y, x^(i-1), x) from the
                        # start of the iteration, under the q that iteration verified against
                        _memo[block] = residual_literal(p_rel, q_rel, block[n0:], V, K)[0]
                    else:
                        Qj, Pj = joint(q_rel, _key), joint(p_rel, _key)
                        for i in range(len(_np), len(block)):
                            Qj *= q_of(block[:i])[block[i]]
                            Pj *= p_of(block[:i])[block[i]]
                        wts = [Qj * q_of(block)[x] * _one_minus_min_pow(Pj * p_of(block)[x], Qj * q_of(block)[x], K)
                               for x in range(V)]
                        tot = sum(wts)
                        _memo[block] = [v / tot for v in wts] if tot != 0 else list(q_of(block))
                return _memo[block]

            run(new_prefix, pr * w, new_target, it + 1)

    run((), Fraction(1), q_of, 0)
    assert sum(out.values()) == 1
    return out


def first_token_marginal(dist, V: int):
    m = [Fraction(0)] * V
    for key, pr in dist.items():
        m[key[0]] += pr
    return m


def table_from_dict(d):
    """Table callable from {block tuple: [Fraction,...]}."""
    return lambda block: d[tuple(block)]


def random_tables(rng, V: int, L: int, denom: int = 12):
    """Strictly positive random rational conditional tables for all blocks of length <= L."""
    def rand_dist():
        while True:
            cuts = sorted(rng.integers(1, denom, size=V - 1).tolist())
            parts = [a - b for a, b in zip(cuts + [denom], [0] + cuts)]
            if all(v > 0 for v in parts):
                return [Fraction(v, denom) for v in parts]
    p, q = {}, {}
    for r in range(L + 1):
        for block in itertools.product(range(V), repeat=r):
            p[block] = rand_dist()
            q[block] = rand_dist()
    return table_from_dict(p), table_from_dict(q)


# ---------------------------------------------------------------------------
# SpecTr K-SEQ (Section 3.2): brute force in float64 (rho is the root of a polynomial-like equation and is
# irrational in general, so this part cannot be exact rationals; every other step is a finite enumeration).

def kseq_rho_float(p, q, k: int) -> float:
    """Root of 1 - (1 - beta(rho))^k = rho beta(rho), beta(rho) = sum_x min{p[x], q[x]/rho}, in [1, k]."""
    if k <= 1:
        return 1.0

    def f(rho):
        b = sum(min(float(px), float(qx) / rho) for px, qx in zip(p, q))
        return rho * b - 1.0 + (1.0 - b) ** k

    lo, hi = 1.0, float(k)
    if f(lo) >= 0.0:
        return lo
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if not (lo < mid < hi):
            break
        if f(mid) >= 0.0:
            hi = mid
        else:
            lo = mid
    return hi


def enumerate_kseq(p_of: Table, q_of: Table, V: int, L: int, K: int, retained_reading: bool = True):
    """Law of the K-SEQ procedure's output (Section 3.2) on autoregressive tables, by enumeration of every draft
    tuple and every accept/reject branch.  Returns (dist, E_tau): dist maps the emitted token tuple (accepted
    tokens followed by the residual or bonus token) to its probability.  With retained_reading=False the root is
    taken for k = K at every position instead of the number of drafts still retained (shown by the tests to
    break the output law: this is why the other reading is the one implemented)."""
    dist: Dict[Block, float] = {}
    E_tau = 0.0
    blocks = list(itertools.product(range(V), repeat=L))
    for drafts in itertools.product(blocks, repeat=K):
        pd = 1.0
        for d in drafts:
            pd *= float(joint(p_of, d))
        if pd == 0.0:
            continue

        def rec(i, alive, accepted, pr):
            nonlocal E_tau
            if pr == 0.0:
                return
            if i == L:                                   # every position accepted: bonus token from q(.|x^L)
                qrow = [float(v) for v in q_of(accepted)]
                E_tau += pr * L
                for y in range(V):
                    if qrow[y] > 0:
                        dist[accepted + (y,)] = dist.get(accepted + (y,), 0.0) + pr * qrow[y]
                return
            p = [float(v) for v in p_of(accepted)]
            q = [float(v) for v in q_of(accepted)]
            rho = kseq_rho_float(p, q, len(alive) if retained_reading else K)
            beta = sum(min(p[x], q[x] / rho) for x in range(V))
            none_yet = pr
            for j in alive:                              # candidates in draft order; the first accepted one wins
                x = drafts[j][i]
                a = min(1.0, q[x] / (rho * p[x])) if p[x] > 0 else 1.0
                nxt = tuple(m for m in alive if drafts[m][i] == x)
                rec(i + 1, nxt, accepted + (x,), none_yet * a)
                none_yet *= 1.0 - a
            if none_yet > 0.0:                           # all rejected: residual (q - rho min{p, q/rho}) / (1 - rho beta)
                E_tau += none_yet * i
                norm = 1.0 - rho * beta
                for y in range(V):
                    w = q[y] - rho * min(p[y], q[y] / rho)
                    if w > 0 and norm > 0:
                        dist[accepted + (y,)] = dist.get(accepted + (y,), 0.0) + none_yet * w / norm

        rec(0, tuple(range(K)), (), pd)
    return dist, E_tau
