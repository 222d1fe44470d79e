"""What ANY valid multi-draft verifier can accept at a single position: the optimal coupling, by linear programming.

TEST / DIAGNOSTIC INFRASTRUCTURE (CPU only, like the rest of oracle/).

Setting of Sections 3.2 and 4 for one position (L = 1): K drafts X_1..X_K i.i.d. from p, one output Y that must be
distributed as q.  A verifier is a conditional law of Y given the drafts, i.e. a coupling pi(x_1..x_K, y) with
marginals p^{(x)K} on the drafts and q on the output; it "accepts" when Y is one of the drafts.  The largest
acceptance probability any such verifier can have is the linear program

    maximise   sum_{(x, y): y in {x_1..x_K}} pi(x, y)
    subject to sum_y pi(x, y) = prod_k p(x_k)  for every draft tuple x,   sum_x pi(x, y) = q(y)  for every y,   pi >= 0

(the multi-draft optimal transport problem the SpecTr line of work starts from).  It is solved here with scipy's
HiGHS on tiny vocabularies and set beside three numbers for the same tables:
  * the closed form of Theorem 5.3 at L = 1,  1 - sum_x q(x) max(1 - p(x)/q(x), 0)^K;
  * what Algorithm 1 as printed does (exact enumeration): its acceptance probability and the total-variation distance
    of its output from q -- zero only at K = 1;
  * what the K-SEQ rule of Section 3.2 accepts (exact enumeration; its output is q for every K).
The optimum bounds every distribution-preserving rule from above, so it says how much a corrected K >= 2 rule could
gain at most over K-SEQ, and whether the closed form is within reach of a valid rule at all.

    python -m oracle.optimal_coupling
"""
from __future__ import annotations

import itertools
from fractions import Fraction

import numpy as np


def optimal_acceptance(p, q, K: int) -> float:
    """max over couplings of (X_1..X_K) ~ p i.i.d. and Y ~ q of P(Y in {X_1..X_K})."""
    from scipy.optimize import linprog
    from scipy.sparse import lil_matrix

    p = np.asarray([float(v) for v in p], dtype=np.float64)
    q = np.asarray([float(v) for v in q], dtype=np.float64)
    V = len(p)
    tuples = list(itertools.product(range(V), repeat=K))
    n = len(tuples) * V                                   # variable (t, y) at index t * V + y
    cost = np.zeros(n)
    A = lil_matrix((len(tuples) + V, n))
    b = np.zeros(len(tuples) + V)
    for ti, t in enumerate(tuples):
        b[ti] = float(np.prod(p[list(t)]))
        members = set(t)
        for y in range(V):
            j = ti * V + y
            A[ti, j] = 1.0
            A[len(tuples) + y, j] = 1.0
            if y in members:
                cost[j] = -1.0                            # linprog minimises
    b[len(tuples):] = q
    # the last output marginal follows from the others (both sides have total mass one); leaving it out keeps the
    # system consistent when the float sums of p^K and q differ in the last bit
    A, b = A.tocsr()[:-1], b[:-1]
    res = linprog(cost, A_eq=A, b_eq=b, bounds=(0, None), method="highs")
    if res.status != 0:
        raise RuntimeError("linear program not solved: " + res.message)
    return float(-res.fun)


def optimal_acceptance_min_cut(p, q, K: int) -> float:
    """The same optimum from the max-flow / min-cut theorem on the bipartite graph (draft tuple) -- (output it
    contains): min over sets S of outputs of  q(complement of S) + P(some draft lies in S) = 1 - q(S) + 1 - (1 - p(S))^K.
    Brute force over the 2^V subsets; pins the linear program's value independently of the solver."""
    p = [float(v) for v in p]
    q = [float(v) for v in q]
    V = len(p)
    best = 1.0
    for r in range(1, V + 1):
        for S in itertools.combinations(range(V), r):
            pS, qS = sum(p[x] for x in S), sum(q[x] for x in S)
            best = min(best, 1.0 - qS + 1.0 - (1.0 - pS) ** K)
    return best


def closed_form_single_position(p, q, K: int) -> float:
    """Theorem 5.3 at L = 1: sum_x q(x) [1 - (1 - min{p(x)/q(x), 1})^K]."""
    tot = 0.0
    for px, qx in zip(p, q):
        px, qx = float(px), float(qx)
        if qx > 0.0:
            tot += qx * (1.0 - (1.0 - min(px / qx, 1.0)) ** K)
    return tot


def single_position_table(p, q, Ks=(1, 2, 3)):
    """Rows (K, optimum, closed form, printed algorithm's acceptance, its TV distance from q, K-SEQ's acceptance)."""
    from . import exact_enum as ee

    pf = [Fraction(v).limit_denominator(10 ** 6) for v in p]
    qf = [Fraction(v).limit_denominator(10 ** 6) for v in q]
    V = len(pf)
    p_of = lambda blk: pf
    q_of = lambda blk: qf
    rows = []
    for K in Ks:
        dist, e_tau, _ = ee.enumerate_alg1(p_of, q_of, V, 1, K)
        out = [Fraction(0)] * V                            # law of the one emitted token
        for key, pr in dist.items():
            out[key[0]] += pr
        tv = float(sum(abs(out[y] - qf[y]) for y in range(V)) / 2)
        _, e_kseq = ee.enumerate_kseq(p_of, q_of, V, 1, K)
        rows.append((K, optimal_acceptance(pf, qf, K), closed_form_single_position(pf, qf, K), float(e_tau), tv,
                     float(e_kseq)))
    return rows


def main() -> int:
    cases = [
        ("p = (1/2, 1/2), q = (4/5, 1/5)", [Fraction(1, 2), Fraction(1, 2)], [Fraction(4, 5), Fraction(1, 5)]),
        ("p = q = (1/2, 1/2)", [Fraction(1, 2)] * 2, [Fraction(1, 2)] * 2),
        ("p = (1/2, 1/3, 1/6), q = (1/6, 1/3, 1/2)", [Fraction(1, 2), Fraction(1, 3), Fraction(1, 6)],
         [Fraction(1, 6), Fraction(1, 3), Fraction(1, 2)]),
        ("p = (7/10, 1/10, 1/10, 1/10), q = (1/4, 1/4, 1/4, 1/4)",
         [Fraction(7, 10)] + [Fraction(1, 10)] * 3, [Fraction(1, 4)] * 4),
    ]
    for name, p, q in cases:
        print(name)
        print("| K | optimal coupling | closed form (Thm 5.3) | Algorithm 1 as printed: accepts / TV from q | K-SEQ accepts |")
        print("|---|---|---|---|---|")
        for K, opt, cf, alg, tv, ks in single_position_table(p, q):
            print("| %d | %.6f | %.6f | %.6f / %.6f | %.6f |" % (K, opt, cf, alg, tv, ks))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
