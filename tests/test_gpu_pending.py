"""GPU <-> oracle parity of a verification that applies a pending distribution modification
(Algorithm 2) on the fly, through the C ABI.

Expected values: the oracle's Algorithm 2 on the same rows (float64 log-probabilities), then the
oracle's Algorithm 1 on those rows at temperature 1 -- the composition the on-the-fly path
replaces.  The GPU reads the raw logits and the carried (ratio, count) pair only.  Bar: the one
of the plain verification (decisions and tokens bit-exact except below the 1e-6 margins,
probabilities to 1e-5 relative); the log-normalisers of the target rows are not compared (the
oracle sees normalised rows, the library reports those of the raw rows).

Conditioning.  The modified probability of a drafted token is q'[x] = q[x] t^K / N with
t = 1 - r, r = p[x] / (mu q[x]); any float32 evaluation of the row statistics leaves a relative
error of up to EPS_R = 1e-6 on r, i.e. K EPS_R r / (1 - r) on ln q'[x], which is unbounded as
r -> 1 (such a token has almost no mass under q' and its block is all but never accepted).  That
amount, accumulated along the block, is admitted on ln nu_i on top of the 1e-5 and propagated to
s, h, the residual normaliser and the carried ratio by parity_util.compare; a prefix with a
drafted token within 4 EPS_R of r = 1 (where even the sign of t is undecided) is left out and counted.
"""
import numpy as np
import pytest

import oracle
from parity_util import compare, run_gpu
from specgbv_synth import WORKLOADS, Workload, make_inputs, with_batch

pytestmark = pytest.mark.gpu


def _as_f64(raw):
    if raw.dtype == np.uint16:
        return (raw.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return raw.astype(np.float64)


def _levels(carry, count):
    carry, count = np.asarray(carry, np.float64), np.asarray(count, np.int32)
    return (carry[None], count[None]) if carry.ndim == 1 else (carry, count)


def oracle_pending(t, d, tok, T, seed, offset, carry, count, prefix_ids=None):
    """Algorithm 2 level by level (innermost first), then Algorithm 1 on its rows (all the oracle's),
    without any rounding in between.  Returns the verification's outputs and, per level, what
    oracle.modify returned plus the rows it modified as log-probabilities."""
    carry, count = _levels(carry, count)
    B, K, L1, V = t.shape
    L = L1 - 1
    Tf = float(np.float32(T))                           # the oracle widens the float32 temperature
    dq = _as_f64(d) / Tf
    lnp = np.empty((B, K, L, V), np.float64)
    lnq = np.empty((B, K, L, V), np.float64)
    for b in range(B):
        for k in range(K):
            for r in range(L):
                lnp[b, k, r] = oracle.log_softmax(dq[b, k, r], 1.0)[0]
                lnq[b, k, r] = oracle.log_softmax(_as_f64(t[b, k, r]), Tf)[0]
    mods = []
    cur = lnq
    for l in range(carry.shape[0]):
        if l == 0:
            mod = oracle.modify(np.ascontiguousarray(t[:, :, :L]), d, tok, T, carry[l], count[l])
        else:
            mod = oracle.modify(cur, dq, tok, 1.0, carry[l], count[l])
        mod["lnq_in"] = cur
        mods.append(mod)
        cur = mod["logq"]
    tq = np.empty((B, K, L + 1, V), np.float64)
    tq[:, :, :L] = cur
    tq[:, :, L] = _as_f64(t[:, :, L]) / Tf              # bonus row: plain logits over T, used at temperature 1
    ora = oracle.verify(tq, dq, tok, 1.0, seed, offset, debug=True, nthreads=8, prefix_ids=prefix_ids)
    return ora, mods, lnp


EPS_R = 1e-6


def conditioning(tok, K, carry, count, mods, lnp, ora):
    """(nu_extra [B, K, L], carry_extra [B], undecided [B]) from the oracle's float64 values.  A level
    multiplies a token's probability by t^K / N, t = 1 - r, r = p / (mu q): a relative error e on r
    (EPS_R of the float32 evaluation, plus the errors the token probability and the block ratio
    already carry from the levels and rows before) becomes K e r / (1 - r) on the logarithm.  The
    bounds are accumulated over levels and along each block; a prefix with a drafted token within
    4 EPS_R of r = 1 at some level (even the sign of t is undecided there) is reported separately."""
    carry, count = _levels(carry, count)
    B, _, L = tok.shape
    nu_extra = np.zeros((B, K, L))
    carry_extra = np.zeros(B)
    undecided = np.zeros(B, bool)
    for b in range(B):
        tau, kf = int(ora["accepted_len"][b]), max(int(ora["accepted_draft_idx"][b]), 0)
        for k in range(K):
            e_tok = np.zeros(L)                          # error bound of ln q^(l)[token] per row, level by level
            e_y = 0.0                                    # the same for the final token (row tau of draft kf)
            for l, mod in enumerate(mods):
                ln_mu, e_mu = float(carry[l, b]), 0.0
                for j in range(min(int(count[l, b]), L)):
                    x = int(tok[b, k, j])
                    lq, lp = mod["lnq_in"][b, k, j], lnp[b, k, j]
                    if not mod["fallback"][b, k, j]:
                        if k == kf and j == tau and tau < L:
                            y = int(ora["out_tokens"][b, tau])
                            ry = np.exp(lp[y] - lq[y] - ln_mu)
                            if ry < 1.0:
                                e_y += K * (EPS_R + e_y + e_mu) * ry / (1.0 - ry)
                        r = np.exp(lp[x] - lq[x] - ln_mu)
                        if abs(1.0 - r) < 4 * (EPS_R + e_tok[j] + e_mu) * r:
                            undecided[b] = True
                        elif r < 1.0:
                            e_tok[j] += K * (EPS_R + e_tok[j] + e_mu) * r / (1.0 - r)
                    e_mu += e_tok[j] if l > 0 else 0.0
                    ln_mu += lq[x] - lp[x]
            nu_extra[b, k] = np.cumsum(e_tok)
            if k == kf:
                carry_extra[b] = e_y
    return nu_extra, carry_extra, undecided


def check_pending(t, d, tok, T, seed, offset, carry, count, label, gpu_slice=None):
    carry, count = _levels(carry, count)
    pend = (carry[0], count[0]) if carry.shape[0] == 1 else (carry, count)
    gpu = run_gpu(t, d, tok, T, seed, offset, pending=pend)
    if gpu_slice is not None:
        idx = np.asarray(gpu_slice)
        t, d, tok, carry, count = t[idx], d[idx], tok[idx], carry[:, idx], count[:, idx]
        ora, mods, lnp = oracle_pending(t, d, tok, T, seed, offset, carry, count, prefix_ids=idx.astype(np.int32))
        gpu = {k: v[idx] for k, v in gpu.items()}
    else:
        ora, mods, lnp = oracle_pending(t, d, tok, T, seed, offset, carry, count)
    nu_extra, carry_extra, undecided = conditioning(tok, t.shape[1], carry, count, mods, lnp, ora)
    keep = ~undecided
    rep = compare({k: v[keep] for k, v in gpu.items()}, {k: v[keep] for k, v in ora.items()}, tok[keep], label=label,
                  skip=("lse_q",), nu_extra=nu_extra[keep], carry_extra=carry_extra[keep])
    rep["undecided_prefixes"] = int(undecided.sum())
    rep["max_nu_extra"] = float(nu_extra[keep].max()) if keep.any() else 0.0
    assert undecided.sum() <= 1
    print("[parity] %s: %s" % (label, rep), flush=True)
    return rep, gpu, ora, mods[-1] if len(mods) == 1 else mods


@pytest.mark.parametrize("B,K,L,V,dtype,T", [
    (16, 3, 4, 515, "f32", 1.0),          # scalar-load path
    (12, 4, 5, 8192, "bf16", 0.8),
    (16, 1, 3, 4096, "f32", 0.6),         # K = 1: greedy block verification under a modification
    (8, 2, 1, 1000, "f32", 1.0),          # L = 1: nothing to modify (count is 0 or clamped away)
    (6, 8, 8, 32000, "f32", 0.4),
])
def test_pending_verification_matches_oracle(B, K, L, V, dtype, T):
    w = Workload("pend", B, K, L, V, dtype, 2.5, 0.8, head=20, temperature=T)
    t, d, tok = make_inputs(w, seed=61)
    rng = np.random.default_rng(7)
    carry = rng.normal(1.5, 0.8, B)                     # ratios around 4: most drafted tokens keep some mass
    count = rng.integers(0, L + 1, B).astype(np.int32)
    count[0] = 0
    if B > 1:
        count[1] = max(L - 1, 0)
    rep, gpu, ora, mod = check_pending(t, d, tok, T, 5, 3, carry, count, "pending %s V=%d K=%d L=%d" % (dtype, V, K, L))
    assert rep["decision_mismatches"] <= 1 and rep["token_mismatches"] <= 1
    if L > 1:
        assert (mod["norm"][count > 0] < 1.0).any()          # something was really modified
        assert (ora["accepted_len"] > 0).any()


def test_pending_with_zero_count_is_the_plain_verification():
    w = Workload("pend0", 8, 3, 4, 4096, "bf16", 2.5, 0.8, head=20, temperature=0.9)
    t, d, tok = make_inputs(w, seed=62)
    plain = run_gpu(t, d, tok, w.temperature, 9, 1, algo="split")
    pend = run_gpu(t, d, tok, w.temperature, 9, 1, pending=(np.zeros(8), np.zeros(8, np.int32)))
    for k in plain:
        assert np.array_equal(plain[k], pend[k], equal_nan=True), k


def test_pending_all_zero_weights_and_zero_probability_tokens():
    """A carried ratio so small that every weight of a modified row vanishes leaves the row q
    (the oracle's rule); one so that drafted tokens get probability zero under q_new gives
    blocks of likelihood ratio zero, which are never accepted."""
    w = Workload("pendz", 6, 2, 3, 2048, "f32", 2.5, 0.8, head=20, temperature=1.0)
    t, d, tok = make_inputs(w, seed=63)
    carry = np.array([-200.0, -200.0, -3.0, -3.0, 0.0, 40.0])
    count = np.array([2, 1, 2, 3, 2, 2], np.int32)
    rep, gpu, ora, mod = check_pending(t, d, tok, 1.0, 2, 0, carry, count, "pending degenerate")
    assert mod["fallback"][0].any() and mod["fallback"][1, :, 0].all()
    assert np.isneginf(ora["log_nu"]).any()
    assert rep["decision_mismatches"] == 0


def test_pending_cfg4_rows():
    """Full-size rows (V = 128256, bf16, K = L = 8) in the default launch configuration; the
    oracle recomputes two of the prefixes."""
    w = with_batch(WORKLOADS["cfg4"], 4)
    t, d, tok = make_inputs(w, seed=64)
    carry = np.array([0.3, -0.4, 0.0, 1.1])
    count = np.array([3, 7, 1, 5], np.int32)
    rep, gpu, ora, mod = check_pending(t, d, tok, w.temperature, 3, 2, carry, count, "pending cfg4 rows", gpu_slice=[1, 3])
    assert rep["decision_mismatches"] == 0


@pytest.mark.parametrize("B,K,L,V,dtype,T,levels", [
    (12, 3, 5, 2048, "f32", 1.0, 2),
    (8, 4, 6, 8192, "bf16", 0.8, 3),
    (6, 2, 8, 1003, "f32", 0.7, 8),        # scalar-load path
    (4, 2, 12, 2048, "f32", 0.8, 16),      # as many levels as the library takes
])
def test_several_pending_levels_match_oracle(B, K, L, V, dtype, T, levels):
    """Modifications on top of each other (Algorithm 3 updates q in place): level l is Algorithm 2
    applied to the rows as level l - 1 left them."""
    w = Workload("pendl", B, K, L, V, dtype, 2.5, 0.8, head=20, temperature=T)
    t, d, tok = make_inputs(w, seed=71)
    rng = np.random.default_rng(11)
    carry = rng.normal(2.0, 0.8, (levels, B))
    count = rng.integers(0, L, (levels, B)).astype(np.int32)
    count[:, 0] = 0
    rep, gpu, ora, mods = check_pending(t, d, tok, T, 6, 4, carry, count, "pending %d levels %s V=%d K=%d L=%d" % (levels, dtype, V, K, L))
    assert rep["decision_mismatches"] <= 1 and rep["token_mismatches"] <= 1
    assert sum(int((m["norm"] < 1.0).any()) for m in mods) >= 2          # at least two levels really modify rows
    assert (ora["accepted_len"] > 0).any()


@pytest.mark.parametrize("B,K,L,V,dtype,alive", [(33, 5, 8, 3072, "bf16", 0.2), (40, 3, 6, 1531, "f32", 0.06),
                                                  (9, 2, 4, 16384, "bf16", 0.5)])
def test_levels_with_few_rows_left(B, K, L, V, dtype, alive):
    """The level passes share a modified row among as many workgroups as the grid allows for the rows the level
    has left: the higher levels here are alive in a small fraction of the prefixes only, so every pass works with
    another number of parts per row (from one to the maximum), and the parts are ragged (V is not a multiple of
    the part count times the vector width)."""
    w = Workload("pendf", B, K, L, V, dtype, 2.5, 0.8, head=20, temperature=0.9)
    t, d, tok = make_inputs(w, seed=73)
    rng = np.random.default_rng(13)
    levels = min(L - 1, 5)
    carry = rng.normal(1.8, 0.8, (levels, B))
    count = rng.integers(1, L, (levels, B)).astype(np.int32)
    count[1:] *= (rng.random((levels - 1, B)) < alive)
    count[-1, :] = 0
    count[-1, B // 2] = L - 1                     # the last level: one prefix only
    rep, gpu, ora, mods = check_pending(t, d, tok, 0.9, 8, 2, carry, count, "pending, few rows left %s V=%d" % (dtype, V))
    assert rep["decision_mismatches"] <= 1 and rep["token_mismatches"] <= 1


def test_two_pending_levels_cfg4_rows():
    w = with_batch(WORKLOADS["cfg4"], 3)
    t, d, tok = make_inputs(w, seed=72)
    carry = np.array([[0.8, 1.5, 0.2], [1.9, 0.4, 2.5]])
    count = np.array([[2, 6, 0], [5, 3, 7]], np.int32)
    rep, gpu, ora, mods = check_pending(t, d, tok, w.temperature, 3, 2, carry, count, "pending 2 levels cfg4 rows", gpu_slice=[0, 1])
    assert rep["decision_mismatches"] == 0


def _state_tensor(carry, count, B):
    """The pending_state buffer of the C ABI for the given levels."""
    import torch
    import paper_2604_25925_amd as sg
    buf = np.zeros(sg.specgbv_pending_state_bytes(B), np.uint8)
    c, n = sg.pending_state_views(buf, B)
    c[:carry.shape[0]] = carry
    n[:count.shape[0]] = count
    return torch.from_numpy(buf).cuda()


def _read_state(state, B):
    import paper_2604_25925_amd as sg
    c, n = sg.pending_state_views(state.cpu().numpy(), B)
    return c.copy(), n.copy()


@pytest.mark.parametrize("B,K,L,V,dtype,T,algo", [(24, 3, 6, 2048, "f32", 1.0, "auto"), (16, 2, 8, 8192, "bf16", 0.8, "auto"),
                                                   (12, 4, 9, 515, "f32", 0.9, "auto"), (10, 2, 6, 4 * 7 * 512, "f32", 0.9, "chain"),
                                                   (12, 2, 12, 2048, "f32", 1.0, "auto"), (8, 2, 17, 1024, "f32", 1.0, "auto")])
def test_pending_state_is_updated_like_the_oracle_bookkeeping(B, K, L, V, dtype, T, algo):
    """The in-place state (pending_state) after one call: every level advanced along the emitted tokens
    with the oracle's carry_advance on the rows that level modifies, used-up levels dropped, the new
    modification appended; and the call's outputs equal those of the same levels passed read-only."""
    import torch
    import paper_2604_25925_amd as sg
    from parity_util import to_torch
    w = Workload("pends", B, K, L, V, dtype, 2.5, 0.8, head=20, temperature=T)
    t, d, tok = make_inputs(w, seed=81)
    rng = np.random.default_rng(13)
    nlev = 3 if L < 12 else 6
    carry = rng.normal(2.0, 0.8, (nlev, B))
    count = np.sort(rng.integers(1, L, (nlev, B)).astype(np.int32), axis=0)      # alive levels, none empty
    count[:, 0] = 0                                                              # one prefix with nothing pending
    count[1:, 1] = 0                                                             # one with a single level
    state = _state_tensor(carry, count, B)
    tl, dl, tk = to_torch(t), to_torch(d), to_torch(tok)
    acc, f, out, ws = sg.specgbv_verify_ex(tl, dl, tk, T, 8, 5, pending_state=state, algo=algo)
    torch.cuda.synchronize()
    ro = run_gpu(t, d, tok, T, 8, 5, pending=(carry, count), algo=algo)
    acc, f, out = acc.cpu().numpy(), f.cpu().numpy(), out.cpu().numpy()
    assert np.array_equal(acc, ro["accepted_len"]) and np.array_equal(f, ro["accepted_draft_idx"]) and np.array_equal(out, ro["out_tokens"])
    new_carry, new_count = _read_state(state, B)
    # expected bookkeeping, level by level, on the rows each level modifies (float64, from the oracle)
    ora, mods, lnp = oracle_pending(t, d, tok, T, 8, 5, carry, count)
    Tf = float(np.float32(T))
    want_c, want_n = np.zeros((sg.MAX_PENDING, B)), np.zeros((sg.MAX_PENDING, B), np.int32)
    fill = np.zeros(B, int)
    for l, mod in enumerate(mods):
        rows_q = np.ascontiguousarray(mod["lnq_in"])
        c_adv, n_adv = oracle.carry_advance(rows_q, _as_f64(d) / Tf, tok, acc, f, out, 1.0, carry[l].copy(), count[l].copy())
        for b in range(B):
            if n_adv[b] > 0:
                want_c[fill[b], b], want_n[fill[b], b] = c_adv[b], n_adv[b]
                fill[b] += 1
    for b in range(B):
        if ro["modify_count"][b] > 0:
            want_c[fill[b], b], want_n[fill[b], b] = ro["carry_log_nu"][b], ro["modify_count"][b]
            fill[b] += 1
    assert np.array_equal(new_count, want_n)
    assert (want_n[1] > 0).any() and (want_n[2] == 0).any()                      # several levels survive somewhere, levels are dropped somewhere
    fin = np.isfinite(want_c)
    assert np.array_equal(new_carry[~fin], want_c[~fin])
    nu_extra, carry_extra, undecided = conditioning(tok, K, carry, count, mods, lnp, ora)
    tol = 2e-5 + nu_extra.max(axis=(1, 2)) + carry_extra
    err = np.abs(new_carry - want_c)
    err[~fin] = 0.0
    ok = undecided | (err <= tol[None, :]).all(axis=0)
    assert ok.all(), "carried ratios differ: worst %.3g (tolerance %.3g)" % (err.max(), tol.min())
    assert (want_n > 0).sum() > B                                                # the comparison is not vacuous


@pytest.mark.parametrize("dtype,V,K,levels,B,L", [("bf16", 128256, 8, 1, 3, 5), ("bf16", 65536, 3, 3, 3, 5), ("f32", 32000, 8, 2, 3, 5),
                                                  ("f32", 4 * 7 * 512, 2, 2, 3, 5),
                                                  ("f32", 4 * 7 * 512, 8, 2, 41, 3)])   # more chains than compute units
def test_pending_on_the_chain_schedule(dtype, V, K, levels, B, L):
    """The chain schedule applies pending levels by extra sweeps over the on-chip row pair: same bar.  With more
    chains than compute units a workgroup walks several chains of different prefixes one after the other."""
    w = Workload("pendc", B, K, L, V, dtype, 2.5, 0.8, head=20, temperature=0.9)
    t, d, tok = make_inputs(w, seed=91)
    rng = np.random.default_rng(17)
    carry = rng.normal(2.0, 0.8, (levels, B))
    count = rng.integers(1, L, (levels, B)).astype(np.int32)
    count[0, 0] = 0
    gpu_c = run_gpu(t, d, tok, w.temperature, 4, 1, algo="chain", pending=(carry, count))
    gpu_s = run_gpu(t, d, tok, w.temperature, 4, 1, algo="split", pending=(carry, count))
    ora, mods, lnp = oracle_pending(t, d, tok, w.temperature, 4, 1, carry, count)
    nu_extra, carry_extra, undecided = conditioning(tok, K, carry, count, mods, lnp, ora)
    keep = ~undecided
    for name, gpu in (("chain", gpu_c), ("split", gpu_s)):
        rep = compare({k: v[keep] for k, v in gpu.items()}, {k: v[keep] for k, v in ora.items()}, tok[keep],
                      label="pending %s %s V=%d" % (name, dtype, V), skip=("lse_q",), nu_extra=nu_extra[keep],
                      carry_extra=carry_extra[keep])
        print("[parity] pending on %s: %s" % (name, rep), flush=True)


def test_pending_chain_schedule_is_rejected():
    import paper_2604_25925_amd as sg
    import torch
    from parity_util import to_torch
    w = Workload("pendc", 2, 2, 2, 8192, "bf16", 2.5, 0.8, temperature=1.0)
    t, d, tok = make_inputs(w, seed=65)
    pend = (torch.zeros(2, dtype=torch.float64, device="cuda"), torch.ones(2, dtype=torch.int32, device="cuda"))
    with pytest.raises(sg.SpecGBVError):
        sg.specgbv_verify_ex(to_torch(t), to_torch(d), to_torch(tok), 1.0, 0, 0, algo="chain", pending=pend)
