"""GPU <-> oracle parity of the draft-side sampling (Algorithm 3's drafting step) through the C ABI.

Bar: the uniforms are bit-identical; tokens are identical except where the inverse-CDF margin of
either side is below 1e-6 (counted and reported)."""
import numpy as np
import pytest
import scipy.special
import scipy.stats

import oracle
from parity_util import MARGIN, to_torch
from specgbv_synth import WORKLOADS, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def _gpu_sample(z, T, seed, offset, position):
    import torch
    import paper_2604_25925_amd as sg
    zl = to_torch(z)
    tok, ws = sg.specgbv_sample_tokens(zl, T, seed, offset, position)
    torch.cuda.synchronize()
    inter = sg.specgbv_read_sample_intermediates(ws, z.shape[0], z.shape[1])
    return tok.cpu().numpy(), inter


def _check(z, T, seed, offset, position, label):
    tok, inter = _gpu_sample(z, T, seed, offset, position)
    ora = oracle.sample_rows(z, T, seed, offset, position)
    assert np.array_equal(inter["u"], ora["u"]), label + ": uniforms differ"
    low = (inter["margin"] < MARGIN) | (ora["margin"] < MARGIN)
    diff = tok != ora["tokens"]
    assert not np.any(diff & ~low), "%s: %d tokens differ with margins >= 1e-6" % (label, int((diff & ~low).sum()))
    assert np.all((tok >= 0) & (tok < z.shape[1]))
    print("[sampling parity] %s: rows %d, low-margin %d, mismatches %d" % (label, z.shape[0], int(low.sum()), int(diff.sum())),
          flush=True)


@pytest.mark.parametrize("rows,V,dtype,T", [
    (5, 8, "f32", 1.0), (7, 515, "f32", 0.7), (4, 4104, "bf16", 1.0), (33, 2048, "f32", 1.3),
    (3, 70001, "f32", 1.0), (16, 32000, "f32", 0.8), (6, 131072, "bf16", 1.0),
])
def test_sampling_matches_oracle(rows, V, dtype, T):
    rng = np.random.default_rng(rows * 1000 + V)
    z = rng.normal(0, 2.5, (rows, V)).astype(np.float32)
    z[0, : min(V, 40) : 3] = -np.inf
    if dtype == "bf16":
        z = f32_to_bf16_bits(z)
    for position in (0, 5):
        _check(z, T, 11, position + 2, position, "sample %s pos %d" % ((rows, V, dtype, T), position))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sampling_with_whole_segments_masked(dtype):
    # vocabulary padding longer than a 512-entry segment, masked with -inf, at either end and in the middle:
    # such a segment has no finite entry to take its reference exponent from and must weigh nothing
    rng = np.random.default_rng(77)
    rows, V = 12, 16384
    z = rng.normal(0, 2.5, (rows, V)).astype(np.float32)
    z[:, :1100] = -np.inf
    z[::2, 6000:7700] = -np.inf
    z[:, V - 2048:] = -np.inf
    z[3] -= 500.0
    z[4] += 500.0
    if dtype == "bf16":
        z = f32_to_bf16_bits(z)
    for position in (0, 3):
        tok, _ = _gpu_sample(z, 1.0, 5, position, position)
        assert np.all((tok >= 1100) & (tok < V - 2048))
        _check(z, 1.0, 5, position, position, "sample masked segments %s pos %d" % (dtype, position))


def test_sampling_cfg4_draft_rows():
    """The batch * K = 256 draft rows of one position of the benchmark configuration (V = 128256, bf16);
    the oracle recomputes the first 24 of them (its row index is the Philox counter)."""
    w = WORKLOADS["cfg4"]
    rng = np.random.default_rng(0)
    z = f32_to_bf16_bits(rng.normal(0, 3, (w.batch * w.K, w.V)).astype(np.float32))
    tok, inter = _gpu_sample(z, 1.0, 3, 9, 2)
    n = 24
    ora = oracle.sample_rows(z[:n], 1.0, 3, 9, 2)
    low = (inter["margin"][:n] < MARGIN) | (ora["margin"] < MARGIN)
    assert np.array_equal(inter["u"][:n], ora["u"])
    assert np.array_equal(tok[:n][~low], ora["tokens"][~low])
    assert np.all((tok >= 0) & (tok < w.V))


def test_sampling_law_on_the_gpu():
    rng = np.random.default_rng(4)
    V, n = 7, 60000
    zrow = rng.normal(0, 1.5, V).astype(np.float32)
    z = np.tile(zrow, (n, 1))
    tok, _ = _gpu_sample(z, 0.9, 77, 0, 0)
    counts = np.bincount(tok, minlength=V)
    expect = scipy.special.softmax(zrow.astype(np.float64) / np.float64(np.float32(0.9))) * n
    assert scipy.stats.chisquare(counts, expect).pvalue > 1e-4


def test_sampling_argument_errors():
    import torch
    import paper_2604_25925_amd as sg
    z = torch.zeros((4, 64), device="cuda")
    with pytest.raises(sg.SpecGBVError) as ei:
        sg.specgbv_sample_tokens(z, 0.0, 0, 0, 0)
    assert ei.value.status == 1
    with pytest.raises(sg.SpecGBVError) as ei:
        sg.specgbv_sample_tokens(z, 1.0, 0, 0, 0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == 3
    out, _ = sg.specgbv_sample_tokens(torch.zeros((0, 64), device="cuda"), 1.0, 0, 0, 0)
    assert out.numel() == 0
