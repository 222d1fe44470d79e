"""Random sweep of the verification against the oracle: shapes, dtypes, temperatures, logit scales, vocabulary masks,
common offsets, schedules and the shared-rows-0 statement drawn at random from a fixed seed (needs an MI355X: run
with -m gpu).  Same bar as the other parity tests (parity_util.check_case).  Combinations the library refuses
(a schedule that does not support the shape) are skipped inside the sweep.

This sweep is what found, in this order: infinities turned into NaN by the first-order correction for the float32
rounding of the scale, a cancellation threshold for Eq. (hik) that was too tight for rows dominated by a few
entries, float32 normalisers that lose the mass beside a near-certain drafted token, that token's own term of the
Eq. (hik) sum (seed 36), the scale's rounding in the exponent of the ratios behind long blocks of improbable tokens
(seed 39), and a cancellation threshold that did not know the number of drafts (seed 65).  Seeds 11 and 12 were the
first two; 36, 39 and 65 are kept because their cases failed before the fixes."""
import numpy as np
import pytest

from parity_util import check_case
from specgbv_synth import Workload, f32_to_bf16_bits, make_inputs

pytestmark = pytest.mark.gpu


def _case(rng):
    B = int(rng.integers(1, 6)); K = int(rng.integers(1, 10)); L = int(rng.integers(1, 10))
    kind = rng.integers(0, 4)
    if kind == 0: V = int(rng.integers(8, 3000))
    elif kind == 1: V = int(rng.integers(3000, 40000))
    elif kind == 2: V = int(rng.integers(4, 40)) * 1024
    else: V = int(rng.integers(28672 // 8, 9000)) * 8          # long enough for the on-chip schedule
    dtype = "bf16" if rng.random() < 0.5 else "f32"
    T = float(np.exp(rng.uniform(np.log(0.3), np.log(3.0))))
    st = float(rng.uniform(0.5, 5.0)); sd = float(rng.uniform(0.1, 2.5))
    w = Workload("sweep", B, K, L, V, "f32", st, sd, head=int(rng.integers(0, 30)) if V > 100 else 0, temperature=T)
    t, d, tok = make_inputs(w, seed=int(rng.integers(0, 1 << 30)))
    mask = rng.random() < 0.5
    if mask and V > 16:
        for _ in range(int(rng.integers(1, 4))):
            a = int(rng.integers(0, V)); ln = int(rng.integers(1, max(2, min(V // 2, 3000)))); b_ = min(V, a + ln)
            which = rng.integers(0, 3)
            if which in (0, 2): t[..., a:b_] = -np.inf
            if which in (1, 2): d[..., a:b_] = -np.inf
        ok_idx = np.where(np.isfinite(d).all(axis=(0, 1, 2)) & np.isfinite(t[:, :, :L]).all(axis=(0, 1, 2)))[0]
        if len(ok_idx) < 2:
            return None
        bad = ~np.isfinite(np.take_along_axis(d, tok[..., None].astype(np.int64), axis=-1)[..., 0])
        tok[bad] = rng.choice(ok_idx, size=int(bad.sum()))     # (masks are the same for every draft: rows 0 stay shared)
    if rng.random() < 0.2:
        off = float(rng.uniform(-300, 300)); t += off; d += off
    if dtype == "bf16":
        t, d = f32_to_bf16_bits(t), f32_to_bf16_bits(d)
    algo = ["auto", "split", "chain"][int(rng.integers(0, 3))]
    shared = bool(rng.random() < 0.5)
    seed, off_ = int(rng.integers(0, 1000)), int(rng.integers(0, 1000))
    label = "B%d K%d L%d V%d %s T%.2f st%.1f sd%.1f mask%d %s sh%d" % (B, K, L, V, dtype, T, st, sd, mask, algo, shared)
    return t, d, tok, T, seed, off_, algo, label, shared


@pytest.mark.parametrize("seed", [11, 12, 36, 39, 65])
def test_random_sweep(seed):
    import paper_2604_25925_amd as sg
    rng = np.random.default_rng(seed)
    ran = skipped = 0
    for it in range(46):
        c = _case(rng)
        if c is None:
            continue
        t, d, tok, T, s, off, algo, label, shared = c
        try:
            check_case(t, d, tok, T, s, off, algo, "sweep %d/%d %s" % (seed, it, label), shared_row0=shared)
            ran += 1
        except sg.SpecGBVError as e:
            assert e.status == 2, label                       # refused as unsupported (schedule vs shape), nothing else
            skipped += 1
    assert ran >= 25, (ran, skipped)
