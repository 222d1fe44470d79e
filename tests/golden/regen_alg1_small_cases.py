"""Rewrites alg1_small_cases.json from the exact-rational enumeration in oracle/.

Run from the repository root:  python tests/golden/regen_alg1_small_cases.py
Calls only oracle.exact_enum (no GPU code, no product package).
"""
import json
import os
import sys
from fractions import Fraction as F

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", ".."))
from oracle import exact_enum as ee  # noqa: E402


def frac(v):
    return "%d/%d" % (v.numerator, v.denominator)


def case(name, note, p_of, q_of, V, L, Ks):
    out = {"name": name, "note": note, "V": V, "L": L, "K": {}}
    for K in Ks:
        dist, E, deg = ee.enumerate_alg1(p_of, q_of, V, L, K)
        out["K"][str(K)] = {
            "E_tau_algorithm": frac(E),
            "E_tau_closed_form": frac(ee.closed_form_E_tau(p_of, q_of, V, L, K)),
            "first_token_marginal": [frac(v) for v in ee.first_token_marginal(dist, V)],
            "degenerate_residual_mass": frac(deg),
            "h": {" ".join(map(str, bl)): frac(ee.h_literal(p_of, q_of, bl, V, L, K))
                  for r in range(1, L + 1) for bl in __import__("itertools").product(range(V), repeat=r)},
            "output_law": {" ".join(map(str, k)): frac(v) for k, v in sorted(dist.items())},
        }
    return out


half = lambda b: [F(1, 2), F(1, 2)]
ce1_q = lambda b: [F(4, 5), F(1, 5)]
w2 = {(): [F(4, 5), F(1, 5)], (0,): [F(1, 4), F(3, 4)], (1,): [F(1, 2), F(1, 2)]}
for a in range(2):
    for b in range(2):
        w2[(a, b)] = [F(1, 2), F(1, 2)]

doc = {
    "source": "Exact enumeration of Algorithm 1 with the literal Eq. (hik), Eq. (hLk), Eq. (pres) "
              "(paper Section 4.2) in rational arithmetic; written by regen_alg1_small_cases.py.",
    "cases": [
        case("CE1", "V=2, L=1, p=(1/2,1/2), q=(4/5,1/5). K=1 is textbook speculative decoding "
             "(Section 3.1): E[tau]=sum min(p,q)=7/10 and the output is q. For K=2 the hand "
             "derivation is: h(0)=(4/5)(1-(3/8)^2)/(3/4)=11/12, h(1)=(1/5)/(3/4)=4/15, residual puts "
             "all mass on token 0, P(out=1)=(1/2)(4/15)+(1/4)(1/12)(4/15)=5/36.",
             half, ce1_q, 2, 1, (1, 2, 3)),
        case("CE2_L1", "V=2, L=1, p=q uniform. K=1 accepts always.", half, half, 2, 1, (1, 2, 3)),
        case("CE2_L2", "V=2, L=2, p=q uniform.", half, half, 2, 2, (1, 2, 3)),
        case("W2", "V=2, L=2, p uniform everywhere; q(.|())=(4/5,1/5), q(.|0)=(1/4,3/4), q(.|1)=(1/2,1/2). "
             "Hand derivation of h[(0)] at K=2: P=1/2, Q=4/5; sum=(3/5)(1-5/12)^2=49/240; "
             "g=(4/5)(3/8)^2=27/240; h=(49-27)/240 / (3/4-4/5+49/240)=22/37.",
             half, ee.table_from_dict(w2), 2, 2, (1, 2, 3)),
    ],
}
path = os.path.join(os.path.dirname(__file__), "alg1_small_cases.json")
with open(path, "w") as fh:
    json.dump(doc, fh, indent=1)
print("wrote", path)
