"""The K >= 2 gap diagnostic (oracle/gap_report.py) on a small vocabulary (no GPU).

At K = 1 Theorem 5.3 holds for Algorithm 1 as printed, so the Monte-Carlo mean of the accepted length and the
importance-sampled closed form, both taken over the same drafts, must agree within sampling error; for K >= 2 the
closed form is an upper bound the printed algorithm stays below (the exact values on tiny vocabularies are in
tests/golden/alg1_small_cases.json), and the closed form itself grows with K (Remark 5.2).
"""
from oracle.gap_report import gap_table


def test_gap_report_agrees_at_one_draft_and_shows_the_shortfall_beyond():
    w, rows = gap_table("cfg2", prefixes=500, Ks=(1, 2, 4), seed=3, workers=2, V=512)
    by_k = {r["K"]: r for r in rows}
    r1 = by_k[1]
    sigma = (r1["stderr_algorithm"] ** 2 + r1["stderr_closed_form"] ** 2) ** 0.5
    assert abs(r1["E_tau_algorithm"] - r1["E_tau_closed_form"]) < 4.5 * sigma, r1
    assert by_k[1]["E_tau_closed_form"] < by_k[2]["E_tau_closed_form"] < by_k[4]["E_tau_closed_form"] <= w.L
    for K in (2, 4):
        r = by_k[K]
        assert r["E_tau_algorithm"] < r["E_tau_closed_form"] + 3 * (r["stderr_algorithm"] + r["stderr_closed_form"]), r
