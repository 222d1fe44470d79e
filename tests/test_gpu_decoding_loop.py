"""Algorithm 3 on the GPU with table-defined models: draft (specgbv_sample_tokens), verify
(specgbv_verify), modify the next iteration's target rows (specgbv_modify_target), repeat.

With one draft per prefix the decoded text must be distributed exactly as the target model
(Theorem 4.2 applied iteration after iteration); with K >= 2 drafts it follows the law of the
printed algorithm, obtained by enumerating three iterations in exact rationals.  The test checks
the first three decoded tokens of many independent prefixes that share small conditional tables.  The only
host-side work is looking up each row's logits in the tables, i.e. playing the two models."""
import itertools

import numpy as np
import pytest
from scipy.stats import chi2

from oracle import exact_enum as ee

pytestmark = pytest.mark.gpu


def _markov_tables(rng, V):
    # conditionals that depend on the last two tokens only: tables stay tiny at any depth
    p2, q2 = ee.random_tables(rng, V, 2)
    last = lambda block: tuple(block[-2:])
    return (lambda block: p2(last(block))), (lambda block: q2(last(block)))


@pytest.mark.parametrize("V,K,L,fused", [(3, 1, 2, False), (3, 1, 3, False), (3, 1, 4, False), (2, 2, 2, False),
                                           (2, 2, 3, False), (3, 1, 3, True), (3, 1, 4, True), (2, 2, 3, True),
                                           (3, 1, 3, "state"), (3, 1, 4, "state"), (3, 1, 5, "state"), (2, 2, 3, "state")])
def test_three_iterations_decode_the_exact_law(V, K, L, fused):
    """Algorithm 3 updates q in place ("q <- DistributionModification(q, ...)"), so a modification
    made after one iteration is still in force for its remaining positions when the next iteration
    ends early, and the next modification applies on top of it.  The driver below therefore keeps
    up to L - 1 pending modifications per prefix, innermost first: each has its carried block ratio
    (extended along every emitted token with the probabilities of the distribution it modifies:
    specgbv_carry_advance) and its remaining row count, and the rows handed to the verification are
    obtained by applying them one after the other with specgbv_modify_target.  With fused = True the
    outermost pending modification is not written out: the verification applies it on the fly
    (the pending option of specgbv_verify_ex).  With fused = "state" the library does all of it: the
    loop only hands the same pending_state buffer to every verification (no specgbv_modify_target,
    no specgbv_carry_advance, no q_new tensor)."""
    import torch
    import paper_2604_25925_amd as sg
    rng = np.random.default_rng(100 + L + 10 * K)
    n, iters, m = 60000, 3, 3
    p_of, q_of = _markov_tables(rng, V)
    ctx = [c for r in range(3) for c in itertools.product(range(V), repeat=r)]
    row_id = {c: i for i, c in enumerate(ctx)}
    logp = np.log(np.array([[float(v) for v in p_of(c)] for c in ctx])).astype(np.float32)
    logq = np.log(np.array([[float(v) for v in q_of(c)] for c in ctx])).astype(np.float32)
    ids = lambda blocks: np.array([row_id[tuple(b[-2:])] for b in blocks])
    dev = torch.device("cuda")

    text = [() for _ in range(n)]                       # decoded tokens per prefix
    pending = []                                        # [(carry [n] float64, count [n] int32)] on the GPU, innermost first
    state = torch.zeros(sg.specgbv_pending_state_bytes(n), dtype=torch.uint8, device=dev) if fused == "state" else None
    for it in range(iters):
        # ---- drafting: K i.i.d. blocks per prefix, one position at a time
        blocks = [[text[i] for _ in range(K)] for i in range(n)]
        tokens = np.zeros((n, K, L), np.int32)
        d_logits = np.zeros((n, K, L, V), np.float32)
        t_logits = np.zeros((n, K, L + 1, V), np.float32)
        for r in range(L + 1):
            flat = ids([b for bs in blocks for b in bs])
            t_logits[:, :, r] = logq[flat].reshape(n, K, V)
            if r == L:
                break
            d_logits[:, :, r] = logp[flat].reshape(n, K, V)
            rows = torch.from_numpy(np.ascontiguousarray(d_logits[:, :, r].reshape(n * K, V))).to(dev)
            tok, _ = sg.specgbv_sample_tokens(rows, 1.0, 1234, it, r)
            tokens[:, :, r] = tok.cpu().numpy().reshape(n, K)
            blocks = [[b + (int(tokens[i, k, r]),) for k, b in enumerate(bs)] for i, bs in enumerate(blocks)]
        tl = torch.from_numpy(t_logits).to(dev)
        dl = torch.from_numpy(d_logits).to(dev)
        tk = torch.from_numpy(tokens).to(dev)
        # ---- the pending modifications, innermost first; level_rows[l] is what level l modifies
        # (the tables hold normalised probabilities, so their logits are log-probabilities at T = 1)
        if state is not None:
            acc, f, out, ws = sg.specgbv_verify_ex(tl, dl, tk, 1.0, 1234, it, pending_state=state)
            torch.cuda.synchronize()
            tau, out_h = acc.cpu().numpy(), out.cpu().numpy()
            text = [text[i] + tuple(int(v) for v in out_h[i, :tau[i] + 1]) for i in range(n)]
            continue
        level_rows = [tl]
        cur = tl
        on_the_fly = pending[-1] if (fused and pending) else None
        for carry, count in (pending[:-1] if on_the_fly else pending):
            cur = sg.specgbv_modify_target(cur, dl, tk, 1.0, carry, count)["logq"]
            level_rows.append(cur)
        # ---- verification against the modified rows
        if on_the_fly:
            acc, f, out, ws = sg.specgbv_verify_ex(cur, dl, tk, 1.0, 1234, it, pending=on_the_fly)
        else:
            acc, f, out, ws = sg.specgbv_verify(cur, dl, tk, 1.0, 1234, it)
        cptr, nptr = sg.specgbv_workspace_carry(ws, n, K, L, V)
        assert cptr and nptr
        torch.cuda.synchronize()
        inter = sg.specgbv_read_intermediates(ws, n, K, L, V, 0)
        tau, out_h = acc.cpu().numpy(), out.cpu().numpy()
        text = [text[i] + tuple(int(v) for v in out_h[i, :tau[i] + 1]) for i in range(n)]
        assert all(len(t) >= it + 1 for t in text)
        # ---- every pending ratio moves along the emitted tokens; the new modification is outermost
        for lvl, (carry, count) in enumerate(pending):
            sg.specgbv_carry_advance(level_rows[lvl], dl, tk, acc, f, out, 1.0, carry, count)
        pending.append((torch.from_numpy(inter["carry_log_nu"]).to(dev), torch.from_numpy(inter["modify_count"]).to(dev)))
        pending = [pc for pc in pending if bool(pc[1].any())][-(L - 1):] if L > 1 else []
    # ---- the first m decoded tokens against the exact law: the target model's joint law for one draft
    # (Theorem 4.2, iteration after iteration), the enumerated law of the printed algorithm for K >= 2
    if K == 1:
        law = {blk: ee.joint(q_of, blk) for blk in itertools.product(range(V), repeat=m)}
    else:
        law = {}
        for t, pr in ee.enumerate_decoding(p_of, q_of, V, L, K, iters).items():
            law[t[:m]] = law.get(t[:m], 0) + pr
    counts = {}
    for t in text:
        counts[t[:m]] = counts.get(t[:m], 0) + 1
    assert set(counts) <= {b for b, pr in law.items() if pr > 0}
    stat = sum((counts.get(blk, 0) - float(pr) * n) ** 2 / (float(pr) * n) for blk, pr in law.items() if pr > 0)
    dof = sum(1 for pr in law.values() if pr > 0) - 1
    assert stat < chi2.ppf(1 - 1e-6, dof), "chi-squared %.1f on %d degrees of freedom" % (stat, dof)
    # and the draft model's law is clearly different (the test can tell them apart)
    stat_p = sum((counts.get(blk, 0) - float(ee.joint(p_of, blk)) * n) ** 2 / (float(ee.joint(p_of, blk)) * n)
                 for blk in itertools.product(range(V), repeat=m))
    assert stat_p > 10 * chi2.ppf(1 - 1e-6, V ** m - 1)
