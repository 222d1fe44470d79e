"""GPU <-> oracle parity of the distribution modification (Algorithm 2) through the C ABI.

Bar.  The normaliser sum_x w[x] agrees to 1e-5 relative.  Unmodified rows are ln q to 1e-5
absolute.  For a modified row q_new[x] = q[x] t[x]^K / W with t = max(1 - r, 0), r = p/(nu q):
the kernels form r in float32 (one rounding of the exponent's argument, one of the
exponential, one of the constant folded into "1 - r"), so r carries a relative error of up to
EPS_R = 1e-6, and t = 1 - r cancels when r is close to 1.  The test therefore requires the GPU
value to lie between q t_lo^K / W and q t_hi^K / W with t_lo/hi = max(1 - r (1 +- EPS_R), 0),
widened by 2e-5 relative (q and W) and by the rounding of the float32 output format
(1.2e-7 |ln q_new|).  Where t is not small this is the plain 1e-5 relative bar.
"""
import numpy as np
import pytest

import oracle
from parity_util import RTOL, run_gpu, to_torch
from specgbv_synth import WORKLOADS, Workload, make_inputs, with_batch

pytestmark = pytest.mark.gpu

EPS_R = 1e-6


def _gpu_modify(t, d, tok, T, carry, count, want_logp=True):
    import torch
    import paper_2604_25925_amd as sg
    tl, dl, tk = to_torch(t), to_torch(d), to_torch(np.ascontiguousarray(tok, dtype=np.int32))
    cr = torch.from_numpy(np.ascontiguousarray(carry, dtype=np.float64)).cuda()
    ct = torch.from_numpy(np.ascontiguousarray(count, dtype=np.int32)).cuda()
    res = sg.specgbv_modify_target(tl, dl, tk, T, cr, ct, want_logp=want_logp, want_norm=True)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in res.items() if k != "workspace"}


def _check_modify(t, d, tok, T, carry, count, label):
    B, K, M, V = t.shape
    gpu = _gpu_modify(t, d, tok, T, carry, count)
    ora = oracle.modify(t, d, tok, T, carry, count)
    assert np.array_equal(gpu["fallback"], ora["fallback"]), label + ": all-zero-weight rows differ"
    np.testing.assert_allclose(gpu["norm"], ora["norm"], rtol=RTOL, atol=1e-300, err_msg=label + " normaliser")
    worst_plain, worst_mod = 0.0, 0.0
    for b in range(B):
        for k in range(K):
            lognu = float(carry[b])
            for r in range(M):
                z = (t[b, k, r].astype(np.uint32) << 16).view(np.float32) if t.dtype == np.uint16 else t[b, k, r]
                zp = (d[b, k, r].astype(np.uint32) << 16).view(np.float32) if d.dtype == np.uint16 else d[b, k, r]
                lq, _ = oracle.log_softmax(z, T)
                lp, _ = oracle.log_softmax(zp, T)
                g = gpu["logq"][b, k, r].astype(np.float64)
                gp = gpu["logp"][b, k, r].astype(np.float64)
                assert not np.any(np.isnan(g)), "%s: NaN in row %s" % (label, (b, k, r))
                fin = np.isfinite(lp)
                assert np.array_equal(np.isfinite(gp), fin)
                e = np.abs(gp[fin] - lp[fin]) / (RTOL + 1.2e-7 * np.abs(lp[fin]))
                worst_plain = max(worst_plain, float(e.max()))
                if r < count[b] and not ora["fallback"][b, k, r]:
                    W = ora["norm"][b, k, r]
                    with np.errstate(over="ignore", divide="ignore", invalid="ignore"):
                        ratio = np.exp(lp - lq - lognu)
                        ratio = np.where(np.isnan(ratio), np.inf, ratio)         # q = 0: weight 0 (min{p/q, 1} = 1)
                        t_lo = np.clip(1.0 - ratio * (1.0 + EPS_R), 0.0, 1.0)
                        t_hi = np.clip(1.0 - ratio * (1.0 - EPS_R), 0.0, 1.0)
                        q = np.exp(lq)
                        ref = ora["logq"][b, k, r]
                    slack = 2 * RTOL + 1.2e-7 * np.abs(np.where(np.isfinite(ref), ref, 0.0))
                    lo = q * t_lo ** K / W * (1.0 - slack)
                    hi = q * t_hi ** K / W * (1.0 + slack) + 1e-300
                    got = np.exp(g)
                    bad = (got < lo) | (got > hi)
                    assert not bad.any(), "%s row %s: %d entries outside the propagated bound, first x=%d got %.9g in [%.9g, %.9g]" % (
                        label, (b, k, r), int(bad.sum()), int(np.argmax(bad)), got[np.argmax(bad)],
                        lo[np.argmax(bad)], hi[np.argmax(bad)])
                    # where 1 - r does not cancel (t >= 1/4) this is the plain 1e-5 bar
                    big = (t_lo >= 0.25)
                    if big.any():
                        e = np.abs(g[big] - ref[big]) / (RTOL * (1 + K * 4 * EPS_R / RTOL) + 1.2e-7 * np.abs(ref[big]))
                        worst_mod = max(worst_mod, float(e.max()))
                    assert abs(got.sum() - 1.0) < 1e-4
                else:
                    ref = ora["logq"][b, k, r]
                    fin = np.isfinite(ref)
                    assert np.array_equal(np.isfinite(g), fin)
                    e = np.abs(g[fin] - ref[fin]) / (RTOL + 1.2e-7 * np.abs(ref[fin]))
                    worst_plain = max(worst_plain, float(e.max()))
                lognu += lq[tok[b, k, r]] - lp[tok[b, k, r]]
    print("[modify parity] %s: worst error %.3f x tol (plain log-probabilities), %.3f x tol (modified, t >= 1/4)"
          % (label, worst_plain, worst_mod), flush=True)
    assert worst_plain <= 1.0 and worst_mod <= 1.0
    return gpu, ora


@pytest.mark.parametrize("B,K,M,V,dtype,T", [
    (3, 1, 3, 40, "f32", 0.9),          # single draft: norm(max{nu q - p, 0}) of greedy block verification
    (2, 4, 4, 515, "f32", 1.0),         # ragged V (scalar loads)
    (2, 3, 3, 4104, "bf16", 1.0),
    (2, 8, 7, 8192, "bf16", 0.7),
    (1, 64, 2, 64, "f32", 1.0),         # K at its limit
    (2, 2, 5, 70001, "f32", 1.3),       # odd V, several passes of a workgroup
])
def test_modify_matches_oracle(B, K, M, V, dtype, T):
    w = Workload("mod", B, K, M, V, dtype, 2.5, 0.8, temperature=T)
    t, d, tok = make_inputs(w, seed=21)
    t = np.ascontiguousarray(t[:, :, :M])
    rng = np.random.default_rng(5)
    carry = rng.normal(0, 0.7, B)
    count = rng.integers(0, M + 1, B).astype(np.int32)
    count[0] = M                                          # at least one prefix with every row modified
    _check_modify(t, d, tok, T, carry, count, "modify %s" % ((B, K, M, V, dtype, T),))


def test_modify_cfg4_rows():
    """Rows of the benchmark configuration (V = 128256, bf16, K = 8), 2 prefixes."""
    w = with_batch(WORKLOADS["cfg4"], 2)
    t, d, tok = make_inputs(w, seed=0)
    M = w.L - 1
    t = np.ascontiguousarray(t[:, :, :M]); d = np.ascontiguousarray(d[:, :, :M]); tok = np.ascontiguousarray(tok[:, :, :M])
    _check_modify(t, d, tok, w.temperature, np.array([0.4, -1.1]), np.array([M, 3], np.int32), "modify cfg4/B2")


def test_modify_all_zero_weights_and_masks():
    # p == q with carried ratio 1: every weight vanishes, the row stays q;  -inf logits stay -inf
    rng = np.random.default_rng(8)
    B, K, M, V = 2, 2, 2, 96
    t = rng.normal(0, 1.5, (B, K, M, V)).astype(np.float32)
    d = t.copy()
    d[1] += rng.normal(0, 1, (K, M, V)).astype(np.float32)
    t[1, :, :, 80:] = -np.inf
    d[1, :, :, 90:] = -np.inf
    tok = rng.integers(0, 80, (B, K, M)).astype(np.int32)
    gpu, ora = _check_modify(t, d, tok, 1.0, np.array([0.0, 0.2]), np.array([1, 2], np.int32), "zero weights / masks")
    assert ora["fallback"][0, :, 0].all() and not ora["fallback"][1].any()
    assert np.all(np.isneginf(gpu["logq"][1, :, :, 80:]))


def test_two_iterations_carry_through_the_workspace():
    """Iteration 1 (verify) leaves the carried ratio and row count in its workspace; Algorithm 2
    turns the next drafts' target rows into q_new; iteration 2 verifies against them.  Each stage
    is compared with the oracle on the inputs that stage actually received."""
    import torch
    import paper_2604_25925_amd as sg
    w = Workload("iter", 6, 3, 4, 4096, "bf16", 2.5, 0.8, head=20, temperature=0.8)
    t1, d1, tok1 = make_inputs(w, seed=31)
    T = w.temperature
    tl, dl, tk = to_torch(t1), to_torch(d1), to_torch(tok1)
    a, f, o, ws = sg.specgbv_verify(tl, dl, tk, T, 17, 0)
    carry_ptr, count_ptr = sg.specgbv_workspace_carry(ws, w.batch, w.K, w.L, w.V)
    # the drafts of the next iteration (fresh seeded rows standing in for the models' new outputs)
    t2, d2, tok2 = make_inputs(w, seed=32)
    t2l, d2l, tk2 = to_torch(t2), to_torch(d2), to_torch(tok2)
    M = w.L
    mod = sg.specgbv_modify_target(t2l, d2l, tk2, T, carry_ptr, count_ptr, want_logp=True, want_norm=True)
    torch.cuda.synchronize()
    inter = sg.specgbv_read_intermediates(ws, w.batch, w.K, w.L, w.V, 1)
    ora1 = oracle.verify(t1, d1, tok1, T, 17, 0, debug=True)
    same = (a.cpu().numpy() == ora1["accepted_len"]) & (o.cpu().numpy() == ora1["out_tokens"]).all(axis=1)
    assert same.sum() >= w.batch - 1
    assert np.array_equal(inter["modify_count"][same], ora1["modify_count"][same])
    np.testing.assert_allclose(inter["carry_log_nu"][same], ora1["carry_log_nu"][same], rtol=0, atol=2 * RTOL)
    assert (inter["modify_count"] > 0).any()
    # stage 2 against the oracle from the carried values the GPU produced
    ora_mod = oracle.modify(np.ascontiguousarray(t2[:, :, :M]), d2, tok2, T, inter["carry_log_nu"], inter["modify_count"])
    np.testing.assert_allclose(mod["norm"].cpu().numpy(), ora_mod["norm"], rtol=RTOL)
    # stage 3: verification against the modified rows (float32 log-probabilities, temperature 1);
    # the bonus row L is the unmodified target row, converted to log-probabilities by the same call
    tq = mod["logq"].cpu().numpy()
    logp = mod["logp"].cpu().numpy()
    assert tq.shape == (w.batch, w.K, M + 1, w.V)
    z = (t2[:, :, M].astype(np.uint32) << 16).view(np.float32)
    for b in range(w.batch):
        lq, _ = oracle.log_softmax(z[b, 0], T)
        np.testing.assert_allclose(tq[b, 0, M], lq, rtol=0, atol=3e-5)
    from parity_util import check_case
    rep, gpu, ora = check_case(np.ascontiguousarray(tq), np.ascontiguousarray(logp), tok2, 1.0, 17, 1, "auto",
                               "iteration 2 on modified rows")
    assert np.isneginf(tq).any()


@pytest.mark.parametrize("dtype,V,T", [("f32", 515, 1.0), ("bf16", 8192, 0.8), ("f32", 64, 1.0)])
def test_carry_advance_matches_oracle(dtype, V, T):
    import torch
    import paper_2604_25925_amd as sg
    w = Workload("adv", 24, 3, 4, V, dtype, 2.0, 0.7, temperature=T)
    t, d, tok = make_inputs(w, seed=51)
    tl, dl, tk = to_torch(t), to_torch(d), to_torch(tok)
    acc, f, out, ws = sg.specgbv_verify(tl, dl, tk, T, 8, 0)
    rng = np.random.default_rng(3)
    carry0 = rng.normal(0, 0.5, w.batch)
    count0 = rng.integers(0, w.L, w.batch).astype(np.int32)
    carry, count = torch.from_numpy(carry0.copy()).cuda(), torch.from_numpy(count0.copy()).cuda()
    sg.specgbv_carry_advance(tl, dl, tk, acc, f, out, T, carry, count)
    torch.cuda.synchronize()
    want_c, want_n = oracle.carry_advance(t, d, tok, acc.cpu().numpy(), f.cpu().numpy(), out.cpu().numpy(), T, carry0, count0)
    assert np.array_equal(count.cpu().numpy(), want_n)
    live = want_n > 0
    assert live.any() and (~live).any()
    np.testing.assert_allclose(carry.cpu().numpy()[live], want_c[live], rtol=0, atol=(w.L + 1) * RTOL)
    # expired modifications keep their (unused) ratio
    np.testing.assert_array_equal(carry.cpu().numpy()[~live], carry0[~live])
