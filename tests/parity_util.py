"""Shared helpers of the GPU parity tests: run both sides, compare to the stated bar.

Bar (from the benchmark definition): accepted length, draft index and tokens are
bit-exact except where a decision's margin is below 1e-6 (|eta - h| of a performed
test, or the inverse-CDF margin of the final token); such events are counted and
reported.  Probabilities agree to 1e-5 relative: log-normalisers to 1e-5 (1 + |value|),
ln nu and ln P to 1e-5 absolute in the logarithm (= 1e-5 relative on nu and P), the ratio carried
into Algorithm 2 (ln nu_tau plus the final token's two log-probabilities) to 2e-5; the sums s of Eq. (hik)
and the acceptance probabilities h to 1e-5 relative with an absolute floor of 1e-9; the residual
normaliser to 1e-5.  Nothing is added for the conditioning of h: where its numerator nu (s - g) cancels
(nu > 1, s close to g) both sides evaluate Eq. (hik) through a sum of non-negative terms instead.
Only the tests of rows under pending modifications (Algorithm 2 applied on the fly), which pass an
error bound nu_extra of their own for ln nu, have that bound propagated into the tolerance of h.
"""
from __future__ import annotations

import json
import os

import numpy as np

MARGIN = 1e-6
RTOL = 1e-5


def to_torch(a: np.ndarray, device="cuda"):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def run_gpu(target, draft, tokens, T, seed, offset, algo="auto", plain=False, pending=None, shared_row0=False):
    """Run the library on numpy inputs; returns outputs and intermediates as numpy.  `pending` is a
    pair of numpy arrays (carry_log_nu [B], count [B]): a pending modification applied on the fly.
    `shared_row0`: tell the library that rows 0 of a prefix's drafts are copies of one another."""
    import torch
    import paper_2604_25925_amd as sg
    tl, dl, tk = to_torch(target), to_torch(draft), to_torch(np.ascontiguousarray(tokens, dtype=np.int32))
    B, K, L1, V = tl.shape
    L = L1 - 1
    if plain:
        a, f, o, ws = sg.specgbv_verify(tl, dl, tk, T, seed, offset)
    else:
        pend = None
        if pending is not None:
            pend = (torch.from_numpy(np.ascontiguousarray(pending[0], dtype=np.float64)).to(tl.device),
                    torch.from_numpy(np.ascontiguousarray(pending[1], dtype=np.int32)).to(tl.device))
        a, f, o, ws = sg.specgbv_verify_ex(tl, dl, tk, T, seed, offset, algo=algo, pending=pend, shared_row0=shared_row0)
    torch.cuda.synchronize()
    res = {"accepted_len": a.cpu().numpy(), "accepted_draft_idx": f.cpu().numpy(), "out_tokens": o.cpu().numpy()}
    if B > 0:
        dt = 1 if tl.dtype == torch.bfloat16 else 0
        res.update(sg.specgbv_read_intermediates(ws, B, K, L, V, dt))
    return res


def h_input_sensitivity(ora, K, L, nu_extra=None):
    """|h(nu (1 +- 1e-5), s (1 +- 1e-5) +- 1e-9) - h| maximised over the four corners, evaluated
    with the oracle's own h functions: the part of h's error budget that comes from the
    tolerance already granted to its inputs.  nu_extra [B, K, L] widens the tolerance of ln nu_i
    (and, by the same amount, of s_i)."""
    import oracle
    B = ora["h"].shape[0]
    out = np.zeros_like(ora["h"])
    for b in range(B):
        for k in range(K):
            for i in range(1, L + 1):
                ln, lP, h0 = ora["log_nu"][b, k, i - 1], ora["log_P"][b, k, i - 1], ora["h"][b, k, i - 1]
                worst = 0.0
                if not np.isfinite(ln):         # nu = 0 or infinite: h does not move with its inputs
                    continue
                extra = 0.0 if nu_extra is None else float(nu_extra[b, k, i - 1])
                dl = np.log1p(RTOL) + extra
                if i < L:
                    s0 = ora["s"][b, k, i]
                    ds = RTOL * abs(s0) + 1e-9 + extra
                    for sl in (-dl, dl):
                        for ss in (-ds, ds):
                            worst = max(worst, abs(oracle.h_sub(ln + sl, lP, min(max(s0 + ss, 0.0), 1.0), K) - h0))
                else:
                    for sl in (-dl, dl):
                        worst = max(worst, abs(oracle.h_full(ln + sl, lP, K) - h0))
                out[b, k, i - 1] = worst
    return out


def compare(gpu, ora, tokens, label="", skip=(), nu_extra=None, carry_extra=None):
    """Assert the parity bar; returns a report dict with the counted low-margin events.  Fields
    named in `skip` are not compared.  nu_extra [B, K, L] is an additional absolute error admitted on
    ln nu_i (position i-1) by the caller's error analysis; it widens, by the same absolute amount,
    the sum s_i and the residual normaliser, which move by at most |d ln nu| (the derivative of
    sum_x q max(1 - p/(nu q), 0)^K with respect to ln nu is at most sum_x q = 1), and enters the
    propagated tolerance of h.  carry_extra [B] likewise for the ratio carried into Algorithm 2."""
    propagate = nu_extra is not None
    if nu_extra is None:
        nu_extra = np.zeros(tokens.shape)
    if carry_extra is None:
        carry_extra = np.zeros(tokens.shape[0])
    B, K, L = tokens.shape
    rep = {"prefixes": B, "low_margin_decisions": 0, "decision_mismatches": 0, "low_margin_tokens": 0,
           "token_mismatches": 0, "max_err": {}}

    def relerr(name, g, o, atol=0.0, mask=None):
        g = np.asarray(g, dtype=np.float64)
        o = np.asarray(o, dtype=np.float64)
        if mask is not None:
            g, o = g[mask], o[mask]
            if isinstance(atol, np.ndarray):
                atol = atol[mask]
        if g.size == 0:
            return
        assert np.all(np.isfinite(g)), "%s %s: non-finite GPU value" % (label, name)
        err = np.abs(g - o) / (RTOL * np.abs(o) + atol) if np.all(atol > 0) else np.abs(g - o) / (RTOL * np.abs(o))
        worst = float(np.max(err))
        rep["max_err"][name] = worst
        assert worst <= 1.0, "%s %s: error is %.3g x the tolerance (gpu %r, oracle %r)" % (
            label, name, worst, g.flat[int(np.argmax(err))], o.flat[int(np.argmax(err))])

    def abserr(name, g, o, tol):
        g = np.asarray(g, dtype=np.float64)
        o = np.asarray(o, dtype=np.float64)
        # a block through a token of probability exactly zero has an infinite logarithm on both sides
        inf_o = np.isinf(o)
        assert np.array_equal(g[inf_o], o[inf_o]), "%s %s: infinite oracle values not matched" % (label, name)
        g, o = g[~inf_o], o[~inf_o]
        if isinstance(tol, np.ndarray):
            tol = tol[~inf_o]
        assert np.all(np.isfinite(g)), "%s %s: non-finite GPU value" % (label, name)
        worst = float(np.max(np.abs(g - o) / tol)) if g.size else 0.0
        rep["max_err"][name] = worst
        assert worst <= 1.0, "%s %s: error is %.3g x the tolerance" % (label, name, worst)

    if "lse_q" not in skip:
        relerr("lse_q", gpu["lse_q"], ora["lse_q"][:, :, :L], atol=RTOL)
    relerr("lse_p", gpu["lse_p"], ora["lse_p"], atol=RTOL)
    abserr("log_nu", gpu["log_nu"], ora["log_nu"], RTOL + nu_extra)
    abserr("log_P", gpu["log_P"], ora["log_P"], RTOL)
    if L > 1:
        relerr("s", gpu["s"][:, :, 1:], ora["s"][:, :, 1:], atol=1e-9 + nu_extra[:, :, :L - 1])
    # h: 1e-5 |h| + 1e-9, the stated bar.  (A caller that admits an extra error on ln nu -- rows under pending
    # modifications -- gets what that error implies for h, propagated through the oracle's own formula.)
    htol = RTOL * np.abs(ora["h"]) + 1e-9
    if propagate:
        htol = htol + h_input_sensitivity(ora, K, L, nu_extra)
    herr = np.abs(gpu["h"] - ora["h"]) / htol
    assert np.all(np.isfinite(gpu["h"])), label + " h: non-finite GPU value"
    rep["max_err"]["h"] = float(herr.max())
    rep["max_err"]["h_plain"] = float((np.abs(gpu["h"] - ora["h"]) / (RTOL * np.abs(ora["h"]) + 1e-9)).max())
    assert herr.max() <= 1.0, "%s h: error is %.3g x the tolerance at %s" % (
        label, herr.max(), np.unravel_index(int(np.argmax(herr)), herr.shape))
    assert np.array_equal(gpu["eta"], ora["eta"]), label + " acceptance uniforms differ"
    assert np.array_equal(gpu["u_final"], ora["u_final"]), label + " final uniforms differ"

    rep["conditioning_limited_decisions"] = 0
    for b in range(B):
        tested = (ora["state"][b] == 1) | (gpu["state"][b] == 1)
        dist = np.minimum(np.abs(ora["eta"][b] - ora["h"][b]), np.abs(gpu["eta"][b] - gpu["h"][b]))
        low = bool(np.any(dist[tested] < MARGIN))
        # a test whose |eta - h| is inside the propagated tolerance of that h (only where the caller admitted one)
        cond = propagate and bool(np.any((dist < htol[b])[tested]))
        rep["low_margin_decisions"] += int(low)
        same = (gpu["accepted_len"][b] == ora["accepted_len"][b] and
                gpu["accepted_draft_idx"][b] == ora["accepted_draft_idx"][b])
        if not same:
            assert low or cond, "%s prefix %d: (tau, f) = (%d, %d) vs oracle (%d, %d) with every margin >= 1e-6" % (
                label, b, gpu["accepted_len"][b], gpu["accepted_draft_idx"][b], ora["accepted_len"][b],
                ora["accepted_draft_idx"][b])
            rep["decision_mismatches"] += 1
            rep["conditioning_limited_decisions"] += int(not low)
            continue                      # later fields of a diverged prefix are not compared
        assert np.array_equal(gpu["state"][b], ora["state"][b]), "%s prefix %d: test states differ" % (label, b)
        tau = int(ora["accepted_len"][b])
        go, oo = gpu["out_tokens"][b], ora["out_tokens"][b]
        assert np.array_equal(go[:tau], oo[:tau]) and np.all(go[tau + 1:] == -1), \
            "%s prefix %d: accepted tokens / padding differ" % (label, b)
        assert gpu["fallback"][b] == ora["fallback"][b], "%s prefix %d: residual fallback differs" % (label, b)
        if tau < L:
            kf = max(int(ora["accepted_draft_idx"][b]), 0)
            relerr("res_norm[%d]" % b, gpu["res_norm"][b], ora["res_norm"][b],
                   atol=1e-12 + (float(nu_extra[b, kf, tau - 1]) if tau > 0 else 0.0))
        low_tok = ora["margin"][b] < MARGIN or gpu["margin"][b] < MARGIN
        rep["low_margin_tokens"] += int(low_tok)
        if go[tau] != oo[tau]:
            assert low_tok, "%s prefix %d: final token %d vs oracle %d with margins %.3g / %.3g" % (
                label, b, go[tau], oo[tau], gpu["margin"][b], ora["margin"][b])
            rep["token_mismatches"] += 1
        else:
            assert 0 <= go[tau] < 2 ** 31
            # what Algorithm 2 starts from in the next iteration: ln [nu_tau q_tau[y] / p_tau[y]]
            assert gpu["modify_count"][b] == ora["modify_count"][b], "%s prefix %d: modify_count" % (label, b)
            kf = max(int(ora["accepted_draft_idx"][b]), 0)
            abserr("carry_log_nu[%d]" % b, gpu["carry_log_nu"][b:b + 1], ora["carry_log_nu"][b:b + 1],
                   2 * RTOL + (float(nu_extra[b, kf, tau - 1]) if tau > 0 else 0.0) + float(carry_extra[b]))
    worst = {k: v for k, v in rep["max_err"].items() if "[" not in k}
    for name in ("res_norm", "carry_log_nu"):
        vals = [v for k, v in rep["max_err"].items() if k.startswith(name + "[")]
        if vals:
            worst[name] = max(vals)
    rep["max_err"] = worst
    return rep


def check_case(target, draft, tokens, T, seed=0, offset=0, algo="auto", label="", prefix_ids=None,
               gpu_slice=None, nthreads=8, shared_row0=False):
    """GPU vs oracle on one set of inputs.  With gpu_slice (indices into the batch), the GPU
    runs the whole batch and the oracle only the listed prefixes."""
    import oracle
    gpu = run_gpu(target, draft, tokens, T, seed, offset, algo=algo, shared_row0=shared_row0)
    if gpu_slice is not None:
        idx = np.asarray(gpu_slice)
        ora = oracle.verify(target[idx], draft[idx], tokens[idx], T, seed, offset, debug=True,
                            nthreads=nthreads, prefix_ids=idx.astype(np.int32))
        gpu = {k: v[idx] for k, v in gpu.items()}
        tokens = tokens[idx]
    else:
        ora = oracle.verify(target, draft, tokens, T, seed, offset, debug=True, nthreads=nthreads,
                            prefix_ids=prefix_ids)
    rep = compare(gpu, ora, tokens, label=label)
    print("[parity] %s algo=%s: %s" % (label, algo, rep), flush=True)
    log = os.environ.get("SPECGBV_PARITY_LOG")
    if log:
        with open(log, "a") as fh:
            fh.write(json.dumps({"case": label, "algo": algo, **rep}) + "\n")
    return rep, gpu, ora
