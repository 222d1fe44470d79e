"""Pins of the oracle's drafting step (Algorithm 3: K i.i.d. tokens per position) -- CPU only."""
import numpy as np
import scipy.special
import scipy.stats

import oracle


def test_token_is_the_inverse_cdf_of_its_uniform():
    # independent cumulative sums in numpy: the drawn token's interval must contain u
    rng = np.random.default_rng(1)
    rows, V, T = 300, 37, float(np.float32(0.8))
    z = rng.normal(0, 2, (rows, V)).astype(np.float32)
    z[::7, 5:9] = -np.inf                                   # masked entries are never drawn
    res = oracle.sample_rows(z, T, 9, 4, position=3)
    p = scipy.special.softmax(z.astype(np.float64) / T, axis=1)
    cdf = np.cumsum(p, axis=1)
    for r in range(rows):
        y, u = int(res["tokens"][r]), res["u"][r]
        assert u == oracle.uniform(9, 4, r, 2 ** 31 + 3)    # the documented Philox slot
        lo = cdf[r, y - 1] if y > 0 else 0.0
        assert lo - 1e-12 <= u < cdf[r, y] + 1e-12
        assert p[r, y] > 0.0
        assert abs(res["margin"][r] - min(u - lo, cdf[r, y] - u)) < 1e-12


def test_law_of_the_drawn_tokens_is_the_softmax():
    # many rows holding the same distribution: row index is the only thing that varies
    rng = np.random.default_rng(2)
    V, n, T = 6, 200000, 1.0
    z = rng.normal(0, 1.5, V).astype(np.float32)
    res = oracle.sample_rows(np.tile(z, (n, 1)), T, 123, 0, position=0)
    counts = np.bincount(res["tokens"], minlength=V)
    expect = scipy.special.softmax(z.astype(np.float64) / T) * n
    assert scipy.stats.chisquare(counts, expect).pvalue > 1e-4
    # K drafts of one prefix are different rows: their draws are independent
    a, b = res["tokens"][0::2], res["tokens"][1::2]
    joint = np.zeros((V, V))
    np.add.at(joint, (a, b), 1)
    assert scipy.stats.chi2_contingency(joint + 1e-9)[1] > 1e-4


def test_positions_and_offsets_use_distinct_uniforms():
    z = np.zeros((50, 11), np.float32)
    a = oracle.sample_rows(z, 1.0, 5, 0, position=0)["u"]
    b = oracle.sample_rows(z, 1.0, 5, 0, position=1)["u"]
    c = oracle.sample_rows(z, 1.0, 5, 1, position=0)["u"]
    assert not np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(b, c)
    # flat rows: the token is floor(u * V)
    assert np.array_equal(oracle.sample_rows(z, 1.0, 5, 0, position=0)["tokens"], np.floor(a * 11).astype(np.int32))
