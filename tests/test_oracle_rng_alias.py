"""Pins for the oracle's random numbers and alias-table sampler (CPU only)."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = orc.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_counter_layout_of_a_draw():
    # key = seed halves; counter = (draw lo, draw hi, step lo, stream | dist << 8 | step bits 32..47 << 16)
    seed, stream, dist, step, draw = 0x1122334455667788, 2, 5, (0xABCD << 32) | 0x01020304, (7 << 32) | 9
    expect = orc.philox4x32_10([9, 7, 0x01020304, 2 | (5 << 8) | (0xABCD << 16)], [0x55667788, 0x11223344])
    assert np.array_equal(orc.words(seed, stream, dist, step, draw), expect)


def test_words_are_uniform_and_streams_differ():
    w = np.stack([orc.words(42, 1, 0, 3, i) for i in range(20000)])
    # each of the 4 words, top 4 bits: chi-square against uniform over 16 cells
    for col in range(4):
        obs = np.bincount(w[:, col] >> 28, minlength=16)
        assert stats.chisquare(obs).pvalue > 1e-4
    # bit balance over all 128 bits
    bits = np.unpackbits(w.view(np.uint8), axis=1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 0.02)
    assert not np.array_equal(orc.words(42, 1, 0, 3, 0), orc.words(42, 2, 0, 3, 0))
    assert not np.array_equal(orc.words(42, 1, 0, 3, 0), orc.words(42, 1, 1, 3, 0))
    assert not np.array_equal(orc.words(42, 1, 0, 3, 0), orc.words(42, 1, 0, 4, 0))
    assert not np.array_equal(orc.words(42, 1, 0, 3, 0), orc.words(43, 1, 0, 3, 0))


def _pmf_of_table(thresh, alias):
    """Exact distribution a (thresh, alias) table draws from, in fp64."""
    V = len(thresh)
    keep = thresh.astype(np.float64) / 2.0 ** 32
    # a bucket whose threshold saturated keeps itself except for the single word 0xFFFFFFFF
    p = keep.copy()
    np.add.at(p, alias, 1.0 - keep)
    return p / V


@pytest.mark.parametrize("seed,V", [(0, 1), (1, 2), (2, 7), (3, 64), (4, 1000), (5, 4097)])
def test_alias_table_encodes_target_distribution(seed, V):
    rng = np.random.default_rng(seed)
    w = rng.random(V) ** 3 * 10.0
    w[rng.random(V) < 0.2] = 0.0
    if w.sum() == 0:
        w[0] = 1.0
    thresh, alias = orc.alias_build(w)
    pi = w / w.sum()
    p = _pmf_of_table(thresh, alias)
    assert np.all(alias < V)
    assert np.max(np.abs(p - pi)) <= 2.0 ** -32 + 1e-15 * V
    # zero-weight keys: never kept, never an alias target
    zero = np.flatnonzero(w == 0)
    assert np.all(thresh[zero] == 0)
    assert not np.isin(alias[thresh < 0xFFFFFFFF], zero).any()


def test_alias_zipf_three_quarter_power():
    V = 500
    w = (np.arange(1, V + 1, dtype=np.float64) ** -1.0 * 1e6) ** 0.75
    thresh, alias = orc.alias_build(w)
    assert np.max(np.abs(_pmf_of_table(thresh, alias) - w / w.sum())) <= 2.0 ** -31


def test_alias_rejects_bad_weights():
    for bad in ([0.0, 0.0], [1.0, -1.0], [1.0, float("nan")], [float("inf"), 1.0]):
        with pytest.raises(ValueError):
            orc.alias_build(np.array(bad))


def test_conform_draws_follow_pi_chi_square():
    V, n = 48, 1_000_000
    rng = np.random.default_rng(7)
    w = rng.random(V) + 0.05
    w[[3, 17]] = 0.0
    table = orc.alias_build(w)
    keys = orc.sample_conform(table, V, seed=99, dist_id=0, step=5, n=n)
    assert keys.max() < V
    obs = np.bincount(keys, minlength=V)
    assert obs[3] == 0 and obs[17] == 0
    live = w > 0
    chi = stats.chisquare(obs[live], n * w[live] / w.sum())
    assert chi.pvalue > 1e-4
    # against a brute-force inverse-CDF sampler driven by an unrelated generator:
    # two-sample chi-square on the contingency table
    ref = np.searchsorted(np.cumsum(w / w.sum()), np.random.default_rng(1).random(n), side="right")
    ref = np.minimum(ref, V - 1)
    tab = np.stack([obs[live], np.bincount(ref, minlength=V)[live]])
    assert stats.chi2_contingency(tab)[1] > 1e-4


def test_conform_detects_wrong_distribution():
    # the chi-square above has power: the same draws fail against a slightly different pi
    V, n = 48, 1_000_000
    w = np.random.default_rng(7).random(V) + 0.05
    keys = orc.sample_conform(orc.alias_build(w), V, 99, 0, 5, n)
    w2 = w.copy(); w2[0] *= 1.05
    assert stats.chisquare(np.bincount(keys, minlength=V), n * w2 / w2.sum()).pvalue < 1e-4


def test_conform_is_serially_independent():
    V, n = 8, 400_000
    w = np.arange(1, V + 1, dtype=np.float64)
    keys = orc.sample_conform(orc.alias_build(w), V, 5, 0, 0, n)
    tab = np.zeros((V, V))
    np.add.at(tab, (keys[:-1], keys[1:]), 1)
    assert stats.chi2_contingency(tab)[1] > 1e-4


def test_conform_is_a_pure_function_of_seed_step_draw():
    V = 100
    table = orc.alias_build(np.ones(V))
    a = orc.sample_conform(table, V, 1, 0, 7, 1000)
    assert np.array_equal(a[300:400], orc.sample_conform(table, V, 1, 0, 7, 100, draw0=300))
    assert not np.array_equal(a, orc.sample_conform(table, V, 1, 0, 8, 1000))
    assert not np.array_equal(a, orc.sample_conform(table, V, 2, 0, 7, 1000))


def test_uniform_draws():
    V, n = 37, 500_000
    keys = orc.sample_conform(None, V, 3, 1, 2, n)
    assert keys.max() == V - 1 and keys.min() == 0
    assert stats.chisquare(np.bincount(keys, minlength=V)).pvalue > 1e-4
    # a large key space is covered up to its top
    big = orc.sample_conform(None, 4_600_000, 3, 1, 2, 200_000)
    assert big.max() < 4_600_000 and big.max() > 4_500_000
