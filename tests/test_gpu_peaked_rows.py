"""Rows at the two ends where float32 sums are at their weakest, against the oracle (needs an MI355X: -m gpu).

Near-certain tokens.  A drafted token of probability 1 - eps leaves 1 - P and 1 - Q in Eq. (hik) made of the mass
of all the OTHER entries; a normaliser summed in float32 together with the token's weight (which is one) knows that
mass to 6e-8 absolute, i.e. not at all for eps = 1e-6.  The kernels therefore leave the drafted token out of the
float32 sums and add its weight in float64; these cases fail by factors of 10 - 1000 without that.  Every schedule
that computes row statistics is covered: on-chip chains, the two-pass schedule, rows shared among workgroups
(small batches) and the shared rows 0.

Block ratios that hover about one over near-certain tokens.  With nu within a few 1e-3 of one in front of and behind
a row whose drafted token has nearly all the mass, that token's factor 1 - p/(nu q) = 1 - 1/nu_i is a few 1e-4 and
its term is a good part of the row's whole Eq. (hik) sum at K = 1 (at K = 2 where the rest of the row is as small).
A float32 exponential gives that factor to 6e-8 absolute, the sum to 1e-5 - 1e-4: the kernels take the token's term
again in float64.

Tiny block ratios at a temperature whose scale rounds badly.  The kernels scale logits by the float32 c; what its
rounding leaves out (up to 6e-8 relative) multiplies the exponent of every ratio p/(nu q), which for the entries that
matter is about log2 nu: behind a block of improbable tokens (nu = 2^-40) a ratio of 0.8 moves by 1.5e-6 and the
K-th power of the factor 0.2 by 3e-5 at K = 4.  The kernels take that part of the rounding into the ratio's constant.
(With float32 logits the sweep's own rounding of z_p - z_q is of the same size; bf16 differences are exact.)

A draft close to the target, many drafts.  With p nearly q every row has s barely above g once nu exceeds one
(s = g when the two rows agree), at amplifications s/(s - g) of 4 - 16 that are ordinary rather than rare, and the
K-th power passes K times the float32 error of the entries' factors on to s: a K = 9 row with 83 % of its sum in one
entry is 1.3e-6 off, and at s/(s - g) = 6.7 the plain Eq. (hik) was 1.13 x over its bar.  The amplification up to which
the plain sum serves therefore falls with K (cancel_factor).

Runaway block ratios.  A target far surer of the drafted tokens than the draft makes nu grow by orders of magnitude
per position; s and g = (1 - 1/nu)^K then agree to many digits and Eq. (hik) needs nu^2 (s - g) summed term by term.
On the chain schedule those rows go to a follow-up kernel (chains with every row handed over, workgroups that hand
over more rows than one chain has); on the two-pass schedule they get a second sweep, or, where a small batch
leaves the sums in parts, the final-token kernel's workgroups sum them together.
"""
import numpy as np
import pytest

from parity_util import check_case
from specgbv_synth import Workload, f32_to_bf16_bits, make_inputs

pytestmark = pytest.mark.gpu


def _set_probability(row, x, T, prob):
    """Moves logit x of a float32 row so that softmax(row / T)[x] = prob."""
    others = np.delete(row.astype(np.float64), x) / T
    m = others.max()
    lse = m + np.log(np.exp(others - m).sum())
    row[x] = np.float32(T * (lse + np.log(prob / (1.0 - prob))))


def _case(B, K, L, V, T, seed):
    w = Workload("peaked", B, K, L, V, "f32", 2.5, 0.8, head=0, temperature=T)
    return make_inputs(w, seed=seed)


EPS = [(1e-4, 1e-4), (1e-5, 1e-3), (1e-3, 1e-6), (1e-6, 1e-6), (3e-5, 1e-5)]       # (1 - Q, 1 - P) of the drafted token


@pytest.mark.parametrize("algo,dtype,V,B,shared", [
    ("chain", "bf16", 32768, 3, False), ("chain", "f32", 14336, 3, False), ("chain", "bf16", 40960, 3, True),
    ("split", "f32", 3001, 3, False), ("split", "bf16", 32768, 40, False), ("split", "f32", 16384, 1, False),
    ("auto", "bf16", 32768, 2, True)])
@pytest.mark.parametrize("T", [1.0, 0.4])
def test_near_certain_drafted_tokens(algo, dtype, V, B, shared, T):
    K, L = 4, 4
    t, d, tok = _case(B, K, L, V, T, seed=31)
    rng = np.random.default_rng(32)
    for b in range(B):
        eq, ep = EPS[b % len(EPS)]
        # position 0: the rows 0 of a prefix's drafts are copies of one another, and stay so
        x0 = int(tok[b, 0, 0])
        _set_probability(t[b, 0, 0], x0, T, 1.0 - eq)
        _set_probability(d[b, 0, 0], x0, T, 1.0 - ep)
        for k in range(K):
            t[b, k, 0], d[b, k, 0] = t[b, 0, 0], d[b, 0, 0]
            tok[b, k, 0] = x0 if k != 2 else int(rng.integers(0, V))     # one draft starts with an unlikely token
            for r in range(1, L):                                       # deeper positions: draft k keeps its tokens near-certain
                if k % 2 == 0:
                    _set_probability(t[b, k, r], int(tok[b, k, r]), T, 1.0 - eq * (r + 1))
                    _set_probability(d[b, k, r], int(tok[b, k, r]), T, 1.0 - ep / (r + 1))
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    for off in (0, 1):
        check_case(t, d, tok, T, 5, off, algo, "near-certain %s %s V=%d B=%d T=%g sh%d" % (algo, dtype, V, B, T, shared),
                   shared_row0=shared)


@pytest.mark.parametrize("algo,dtype,V,B,shared", [
    ("chain", "bf16", 32768, 3, False), ("chain", "f32", 14336, 2, False), ("chain", "bf16", 40960, 2, True),
    ("split", "bf16", 131, 4, False), ("split", "f32", 3001, 3, False), ("split", "bf16", 32768, 40, False),
    ("split", "f32", 65536, 1, False), ("auto", "bf16", 32768, 2, True)])
@pytest.mark.parametrize("K,T", [(1, 1.0), (1, 0.3), (2, 0.6)])
def test_block_ratio_hovers_about_one_over_near_certain_tokens(algo, dtype, V, B, shared, K, T):
    L = 6
    t, d, tok = _case(B, K, L, V, T, seed=51)
    rng = np.random.default_rng(52 + K)
    small = lambda lo=2e-4, hi=4e-3: float(np.exp(rng.uniform(np.log(lo), np.log(hi))))
    far = (lambda: small(1e-5, 1e-4)) if K > 1 else small               # K = 2: the rest of the target row as small as the term
    for b in range(B):
        for k in range(K):
            for r in range(L):
                if r == 0 and k > 0:                                    # the rows 0 of a prefix's drafts are copies
                    t[b, k, 0], d[b, k, 0], tok[b, k, 0] = t[b, 0, 0], d[b, 0, 0], tok[b, 0, 0]
                    continue
                x = int(tok[b, k, r])
                _set_probability(t[b, k, r], x, T, 1.0 - far())
                _set_probability(d[b, k, r], x, T, 1.0 - small())
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    kw = {"gpu_slice": list(range(0, B, 13))} if B > 8 else {}
    rep, gpu, ora = check_case(t, d, tok, T, 7, 0, algo, "hovering nu %s %s V=%d B=%d K=%d T=%g sh%d" % (algo, dtype, V, B, K, T, shared),
                               shared_row0=shared, **kw)
    # the case is what it claims: on a good part of the rows the drafted token's term is above a tenth of the sum
    ln_nu, s = ora["log_nu"], ora["s"]
    tok_s = np.asarray(tok)[kw["gpu_slice"]] if kw else np.asarray(tok)
    share = np.maximum(-np.expm1(-ln_nu[:, :, 1:]), 0.0) ** K * 0.99 / np.maximum(s[:, :, 1:], 1e-300)
    assert tok_s.shape == ln_nu.shape and int((share > 0.1).sum()) >= share.size // 5, "the case no longer stresses the term"


@pytest.mark.parametrize("algo,dtype,V,B,K,L", [
    ("chain", "bf16", 32768, 2, 4, 8), ("chain", "f32", 14336, 3, 3, 6), ("chain", "bf16", 28672, 90, 8, 4),
    ("split", "bf16", 32768, 1, 4, 6), ("split", "f32", 16384, 2, 3, 5), ("split", "bf16", 131072, 1, 2, 4),
    ("split", "f32", 3001, 1, 2, 4), ("split", "bf16", 262144, 1, 2, 3), ("split", "bf16", 32768, 40, 4, 4),
    ("split", "bf16", 131072, 192, 2, 3)])
def test_block_ratio_runs_away(algo, dtype, V, B, K, L):
    """q(token) = 0.9 against p(token) = 1e-3 at every position: nu gains a factor 900 per row and every sum of
    Eq. (hik) from the second row on cancels against g.  On the chain schedule B * K = 720 chains on 256 compute
    units make a workgroup hand over the rows of several chains; on the two-pass schedule the small batches leave
    the sums in parts, and the final-token kernel's workgroups find the rows and sum E together (one, four, sixteen
    and thirty-two workgroups per prefix at these vocabularies: the last sixteen only wait); so do the larger
    batches, the last one with 192 x 16 final-token workgroups, more than the chip holds at once."""
    T = 1.0
    t, d, tok = _case(B, K, L, V, T, seed=41)
    for b in range(B):
        for k in range(K):
            if (b + k) % 3 == 2:
                continue                                               # every third chain stays ordinary
            for r in range(L):
                x = int(tok[b, k, r])
                _set_probability(t[b, k, r], x, T, 0.9)
                _set_probability(d[b, k, r], x, T, 1.0e-3)
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    kw = {}
    if B > 8:                                                          # the oracle takes a sample of the prefixes
        kw["gpu_slice"] = list(range(0, B, 11))
    rep, gpu, ora = check_case(t, d, tok, T, 9, 0, algo, "runaway nu %s %s V=%d B=%d" % (algo, dtype, V, B), **kw)
    s, g_ = ora["s"][:, :, 1:], None
    nu = np.exp(np.clip(ora["log_nu"][:, :, :L - 1], -700, 700))
    g_ = np.where(nu > 1, (1 - 1 / np.maximum(nu, 1)) ** K, 0.0)
    assert int(((nu > 1) & ((s - g_) * 16 < s)).sum()) >= s.size // 3, "the case no longer cancels"


def test_bounded_wait_falls_back_to_the_waiting_workgroups_own_sum(monkeypatch):
    """With no look at all at the parts other workgroups sum (SPECGBV_EXCESS_POLLS=0) every workgroup of the
    final-token kernel sums every part of a row that needs E itself: the path a workgroup takes when a part does not
    arrive in time.  Same inputs as above, sixteen workgroups per prefix; the results do not change."""
    monkeypatch.setenv("SPECGBV_EXCESS_POLLS", "0")
    test_block_ratio_runs_away("split", "bf16", 131072, 1, 2, 4)
    test_block_ratio_runs_away("split", "f32", 16384, 2, 3, 5)


def _worst_temperature():
    """The float32 temperature in [0.30, 0.35] whose scale log2(e)/T is furthest from its float32 value."""
    Ts = np.linspace(0.30, 0.35, 400).astype(np.float32)
    c_true = np.log2(np.e) / Ts.astype(np.float64)
    c_rel = c_true / c_true.astype(np.float32).astype(np.float64) - 1.0
    j = int(np.argmax(np.abs(c_rel)))
    return float(Ts[j]), float(c_rel[j])


def _softmax64(row, T):
    z = row.astype(np.float64) / T
    z -= z.max()
    e = np.exp(z)
    return e / e.sum()


@pytest.mark.parametrize("algo,dtype,V,B", [
    ("chain", "bf16", 32768, 3), ("chain", "f32", 14336, 2), ("split", "f32", 3001, 2), ("split", "bf16", 32768, 1),
    ("split", "bf16", 65536, 30)])
def test_tiny_block_ratios_at_a_temperature_whose_scale_rounds_badly(algo, dtype, V, B):
    K, L = 4, 6
    T, c_rel = _worst_temperature()
    assert abs(c_rel) > 4.0e-8
    # float32 logits: their difference z_p - z_q (about 10 here) is itself rounded in the sweep, 6e-8 relative, which
    # this construction amplifies just as much; a ratio of 0.5 keeps that below the bar and the scale's part above it
    ratio = 0.8 if dtype == "bf16" else 0.5
    t, d, tok = _case(B, K, L, V, T, seed=61)
    if dtype == "bf16":                                                 # work on values the kernels will see
        from specgbv_synth import bf16_bits_to_f32
        rnd = lambda a: bf16_bits_to_f32(f32_to_bf16_bits(a))
        t, d = rnd(t), rnd(d)
    else:
        rnd = lambda a: a
    for b in range(B):
        for k in range(K):
            if k > 0:
                t[b, k, 0], d[b, k, 0], tok[b, k, 0] = t[b, 0, 0], d[b, 0, 0], tok[b, 0, 0]
            ln_nu = 0.0
            for r in range(L):
                x = int(tok[b, k, r])
                if r > 0 or k == 0:
                    _set_probability(t[b, k, r], x, T, 1.0e-4)          # improbable under the target,
                    _set_probability(d[b, k, r], x, T, 0.5)             # likely under the draft: nu shrinks by 2^-12 a row
                    t[b, k, r, x], d[b, k, r, x] = rnd(t[b, k, r, x:x + 1])[0], rnd(d[b, k, r, x:x + 1])[0]
                if r >= 2:
                    # one entry y with a tenth of the target's mass and p[y] = ratio nu q[y]: the rest of the row has
                    # p/(nu q) far above one, so the Eq. (hik) sum is q[y] (1 - ratio)^K
                    y = (x + 1 + 7 * r) % V
                    _set_probability(t[b, k, r], y, T, 0.1)
                    t[b, k, r, y] = rnd(t[b, k, r, y:y + 1])[0]
                    q = _softmax64(t[b, k, r], T)
                    _set_probability(d[b, k, r], y, T, min(ratio * np.exp(ln_nu) * q[y], 0.4))
                    d[b, k, r, y] = rnd(d[b, k, r, y:y + 1])[0]
                q, p = _softmax64(t[b, k, r], T), _softmax64(d[b, k, r], T)
                ln_nu += np.log(q[x]) - np.log(p[x])
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    kw = {"gpu_slice": list(range(0, B, 7))} if B > 8 else {}
    rep, gpu, ora = check_case(t, d, tok, T, 3, 0, algo, "tiny nu %s %s V=%d B=%d T=%.6f" % (algo, dtype, V, B, T), **kw)
    front = ora["log_nu"][:, :, 1:L - 1]                                # in front of rows 2 .. L-1
    s = ora["s"][:, :, 2:]
    assert (front < -14.0).all() and ((s > 1e-6) & (s < 1e-2)).mean() > 0.7, "the case no longer is what it claims"


@pytest.mark.parametrize("algo,dtype,V,B,K,L,T", [
    ("split", "f32", 29049, 5, 9, 9, 0.48), ("chain", "bf16", 32768, 4, 8, 8, 0.5), ("auto", "bf16", 16384, 2, 16, 6, 0.6),
    ("chain", "f32", 14336, 6, 6, 8, 0.45)])
def test_draft_close_to_the_target_with_many_drafts(algo, dtype, V, B, K, L, T):
    w = Workload("aligned", B, K, L, V, "f32", 0.8, 0.1, head=0, temperature=T)
    t, d, tok = make_inputs(w, seed=71)
    for b in range(B):                                                  # a first token the target likes better: nu = 2.5 from row 1 on
        x0 = int(tok[b, 0, 0])
        _set_probability(t[b, 0, 0], x0, T, 0.5)
        _set_probability(d[b, 0, 0], x0, T, 0.2)
        for k in range(K):
            t[b, k, 0], d[b, k, 0], tok[b, k, 0] = t[b, 0, 0], d[b, 0, 0], x0
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    rep, gpu, ora = check_case(t, d, tok, T, 11, 0, algo, "aligned %s %s V=%d B=%d K=%d T=%g" % (algo, dtype, V, B, K, T))
    nu = np.exp(np.clip(ora["log_nu"][:, :, :L - 1], -700, 700))
    s = ora["s"][:, :, 1:]
    g = np.where(nu > 1, (1 - 1 / np.maximum(nu, 1)) ** K, 0.0)
    amp = s / np.maximum(s - g, 1e-300)
    assert int(((nu > 1) & (amp > 3) & (amp < 16)).sum()) >= 10, "the case no longer has rows between the two thresholds"
