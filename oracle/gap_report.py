"""How far Algorithm 1 as printed falls short of the paper's closed form for K >= 2, on benchmark-shaped inputs.

TEST / DIAGNOSTIC INFRASTRUCTURE (CPU only, like the rest of oracle/).

Theorem 5.3 states E[tau] = sum_{i=1..L} sum_{x^i} q(x^i) [1 - (1 - min{p(x^i)/q(x^i), 1})^K].  By exact enumeration
on tiny vocabularies (tests/golden/alg1_small_cases.json) the printed Algorithm 1 attains this only at K = 1; this
script measures the gap where enumeration is impossible.  With drafts x ~ p the inner sum is an expectation under p,
    sum_{x^i} q(x^i) [...] = E_{x^i ~ p}[ f_K(nu_i) ],   f_K(nu) = nu (1 - (1 - min{1/nu, 1})^K),   nu_i = q(x^i)/p(x^i),
so the closed form is estimated from the very drafts the algorithm verifies (every draft of every prefix is one
sample; f_K <= min{nu, K} keeps the estimator's variance small), next to the Monte-Carlo mean of the accepted
length the oracle's literal Algorithm 1 produces on them.  At K = 1 the two must agree within sampling error
(Theorem 5.3 holds there); for K >= 2 the difference is what the competition between blocks of different drafts
costs (see the readings in the design notes).

    python -m oracle.gap_report [workload] [prefixes] [workers]
"""
from __future__ import annotations

import sys
from concurrent.futures import ProcessPoolExecutor
from dataclasses import replace

import numpy as np

from specgbv_synth import WORKLOADS, make_prefix


def _job(args):
    w, seed, b = args
    return make_prefix(w, seed, b)


def gap_table(name: str = "cfg2", prefixes: int = 200, Ks=(1, 2, 3, 5, 8), seed: int = 7, workers: int = 8,
              V: int = 0):
    import oracle
    base = WORKLOADS[name]
    Kmax = max(Ks)
    w = replace(base, batch=prefixes, K=Kmax, V=V or base.V)
    store = np.uint16 if w.dtype == "bf16" else np.float32
    t = np.empty((prefixes, Kmax, w.L + 1, w.V), dtype=store)
    d = np.empty((prefixes, Kmax, w.L, w.V), dtype=store)
    tok = np.empty((prefixes, Kmax, w.L), dtype=np.int32)
    jobs = [(w, seed, b) for b in range(prefixes)]
    if workers > 1:
        with ProcessPoolExecutor(max_workers=workers) as ex:
            for b, (tt, dd, kk) in enumerate(ex.map(_job, jobs, chunksize=4)):
                t[b], d[b], tok[b] = tt, dd, kk
    else:
        for b, j in enumerate(jobs):
            t[b], d[b], tok[b] = _job(j)
    rows = []
    for K in Ks:
        tk, dk, kk = np.ascontiguousarray(t[:, :K]), np.ascontiguousarray(d[:, :K]), np.ascontiguousarray(tok[:, :K])
        taus = []
        res = None
        for off in range(4):                                   # four independent sets of uniforms per prefix
            res = oracle.verify(tk, dk, kk, w.temperature, 11, off, debug=True, nthreads=workers)
            taus.append(res["accepted_len"].astype(np.float64))
        tau = np.concatenate(taus)
        nu = np.exp(np.clip(res["log_nu"], -700, 700))         # [B, K, L]: nu_i of every draft
        f = np.where(nu <= 1.0, nu, nu * (1.0 - (1.0 - 1.0 / np.maximum(nu, 1.0)) ** K))
        per_draft = f.sum(axis=2).reshape(-1)                  # one sample of the closed form per draft
        rows.append({"K": K, "E_tau_algorithm": float(tau.mean()), "stderr_algorithm": float(tau.std(ddof=1) / np.sqrt(tau.size)),
                     "E_tau_closed_form": float(per_draft.mean()),
                     "stderr_closed_form": float(per_draft.std(ddof=1) / np.sqrt(per_draft.size)),
                     "samples": int(tau.size)})
    return w, rows


def main(argv):
    name = argv[1] if len(argv) > 1 else "cfg2"
    n = int(argv[2]) if len(argv) > 2 else 200
    workers = int(argv[3]) if len(argv) > 3 else 8
    w, rows = gap_table(name, n, workers=workers)
    print("| K | E[tau], Algorithm 1 as printed | closed form of Theorem 5.3 | ratio |")
    print("|---|---|---|---|")
    for r in rows:
        print("| %d | %.3f +- %.3f | %.3f +- %.3f | %.3f |" % (
            r["K"], r["E_tau_algorithm"], r["stderr_algorithm"], r["E_tau_closed_form"], r["stderr_closed_form"],
            r["E_tau_algorithm"] / r["E_tau_closed_form"]))
    print("(%s-shaped inputs: %d prefixes, L=%d, V=%d, T=%g, four sets of uniforms each)" % (name, n, w.L, w.V, w.temperature))


if __name__ == "__main__":
    main(sys.argv)
