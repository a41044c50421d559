"""Pins for the oracle's sampling schemes (Section 4.4) against the conformity
levels of Section 4.1 and the paper's worked pool-reuse example (CPU only)."""
import os
from collections import Counter

import numpy as np
import pytest
from scipy import stats

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _table(V, seed=0):
    w = np.random.default_rng(seed).random(V) + 0.1
    return w, orc.alias_build(w)


def test_bounded_reproduces_the_papers_worked_example():
    lines = dict((l.split()[0], l.split()[1:]) for l in open(os.path.join(GOLDEN, "pool_reuse_example.txt"))
                 if l.strip() and l[0] != "#")
    U = int(lines["U"][0])
    V = 1000
    w, table = _table(V)
    k = orc.sample_conform(table, V, seed=11, dist_id=0, step=4, n=3)       # the three i.i.d. draws
    assert len(set(k)) == 3
    seq1 = orc.sample_bounded(table, V, 11, 0, 4, n=6, U=U, G=1)
    assert [int(x) for x in seq1] == [int(k[int(i) - 1]) for i in lines["G1"]]
    seq3 = orc.sample_bounded(table, V, 11, 0, 4, n=6, U=U, G=3)
    assert sorted(seq3[:3]) == sorted(k) and sorted(seq3[3:]) == sorted(k)


@pytest.mark.parametrize("N,U,G", [(1000, 4, 16), (1000, 16, 250), (999, 4, 7), (50, 8, 250), (7, 3, 2), (5, 1, 3)])
def test_bounded_invariants(N, U, G):
    V = 100_000                      # large enough that fresh draws are distinct with high probability
    table = orc.alias_build(np.ones(V))
    F = -(-N // U)
    fresh = orc.sample_conform(table, V, 21, 2, 9, F)
    if len(set(fresh)) != F:
        pytest.skip("fresh draws collide for this seed")
    seq = orc.sample_bounded(table, V, 21, 2, 9, N, U, G)
    assert len(seq) == N
    uses = Counter(int(x) for x in seq)
    assert set(uses) <= set(int(x) for x in fresh)
    assert max(uses.values()) <= U                                   # reuse count is bounded by U
    pos = 0
    for first in range(0, F, G):                                     # pool by pool
        pool = sorted(int(x) for x in fresh[first:first + G])
        g = len(pool)
        for r in range(U):                                           # every full pass is a permutation of the pool
            chunk = seq[pos:pos + g]
            if len(chunk) == g:
                assert sorted(int(x) for x in chunk) == pool
            else:
                assert set(int(x) for x in chunk) <= set(pool) and len(set(chunk)) == len(chunk)
            pos += len(chunk)
    assert pos == N
    # all uses of one fresh draw lie within a window of U*G positions
    where = {}
    for i, x in enumerate(seq):
        where.setdefault(int(x), []).append(i)
    assert all(max(v) - min(v) < U * G for v in where.values())
    # every draw of a fully emitted pool is used exactly U times
    full = (N // (U * G)) * G
    assert all(uses[int(x)] == U for x in fresh[:full])


def test_bounded_passes_are_differently_ordered():
    V = 100_000
    table = orc.alias_build(np.ones(V))
    seq = orc.sample_bounded(table, V, 3, 0, 0, 4 * 250, 4, 250)
    passes = seq.reshape(4, 250)
    for a in range(4):
        for b in range(a + 1, 4):
            assert not np.array_equal(passes[a], passes[b])
    fresh = orc.sample_conform(table, V, 3, 0, 0, 250)
    assert not np.array_equal(passes[0], fresh)


def test_bounded_first_order_frequencies_match_pi():
    V = 16
    w, table = _table(V, 3)
    obs = np.zeros(V)
    for step in range(300):
        obs += np.bincount(orc.sample_bounded(table, V, 5, 0, step, 2048, 4, 64), minlength=V)
    # each fresh draw is used 4 times: the chi-square statistic of the counts is inflated 4-fold
    chi = ((obs - obs.sum() * w / w.sum()) ** 2 / (obs.sum() * w / w.sum())).sum() / 4.0
    assert stats.chi2.sf(chi, V - 1) > 1e-4


@pytest.mark.parametrize("P", [1, 2, 3, 5, 16, 17, 64, 1000, 4097])
def test_keyed_permutation_is_a_bijection(P):
    img = [orc.permute(x, P, 77, 1, 2, 3) for x in range(P)]
    assert sorted(img) == list(range(P))
    if P >= 64:
        assert img != list(range(P))
        other = [orc.permute(x, P, 77, 1, 2, 4) for x in range(P)]
        assert other != img
        assert [orc.permute(x, P, 77, 1, 3, 3) for x in range(P)] != img


def test_keyed_permutation_scatters_positions():
    P = 4096
    img = np.array([orc.permute(x, P, 5, 0, 0, 0) for x in range(P)])
    # image of the first quarter is spread over all four quarters
    obs = np.bincount(img[:P // 4] // (P // 4), minlength=4)
    assert stats.chisquare(obs).pvalue > 1e-4
    # neighbours do not stay neighbours
    assert np.mean(np.abs(np.diff(img.astype(np.int64))) < 16) < 0.05


def test_longterm_is_repeated_passes_over_one_pool_then_a_new_pool():
    V, P, R = 50_000, 200, 3
    table = orc.alias_build(np.ones(V))
    seq = orc.sample_longterm(table, V, 9, 1, P, R, cursor=0, n=2 * P * R)
    pool0 = sorted(orc.sample_conform(table, V, 9, 1, step=0, n=P))
    pool1 = sorted(orc.sample_conform(table, V, 9, 1, step=1, n=P))
    assert pool0 != pool1
    for r in range(R):
        assert sorted(seq[r * P:(r + 1) * P]) == pool0
        assert sorted(seq[(R + r) * P:(R + r + 1) * P]) == pool1
    assert not np.array_equal(seq[:P], seq[P:2 * P])


def test_longterm_cursor_continues_across_handles():
    V, P, R = 1000, 77, 2
    w, table = _table(V, 1)
    whole = orc.sample_longterm(table, V, 4, 0, P, R, 0, 500)
    parts = [orc.sample_longterm(table, V, 4, 0, P, R, c, n) for c, n in ((0, 120), (120, 1), (121, 379))]
    assert np.array_equal(whole, np.concatenate(parts))


def test_longterm_long_run_frequencies_match_pi():
    # Eq. (1): relative frequencies converge to pi because the pool is replaced
    V, P, R = 12, 64, 2
    w, table = _table(V, 5)
    n = P * R * 3000
    obs = np.bincount(orc.sample_longterm(table, V, 8, 0, P, R, 0, n), minlength=V)
    chi = ((obs - n * w / w.sum()) ** 2 / (n * w / w.sum())).sum() / R
    assert stats.chi2.sf(chi, V - 1) > 1e-4
    # and it is not the degenerate "one draw used forever" scheme
    assert len(set(orc.sample_longterm(table, V, 8, 0, P, R, 0, 1000))) == V


def test_nonconform_samples_only_keys_of_the_batch_and_follows_their_frequencies():
    B, K = 4096, 5
    ctx = np.random.default_rng(0).zipf(1.5, B).astype(np.uint32) % 1000
    s = orc.sample_nonconform(ctx, ctx, per_example=K, split=K, T=B, seed=3, dist_id=0, step=1, n=B * K)
    assert set(s) <= set(ctx)
    keys, cnt = np.unique(ctx, return_counts=True)
    obs = np.array([np.sum(s == k) for k in keys])
    big = cnt >= 20
    assert stats.chisquare(np.append(obs[big], obs[~big].sum()),
                           B * K * np.append(cnt[big], cnt[~big].sum()) / B).pvalue > 1e-4


def test_nonconform_tiles_and_roles():
    B, K, T = 100, 4, 32
    a = np.arange(B, dtype=np.uint32)                 # key identifies the example it came from
    b = a + 1000
    s = orc.sample_nonconform(a, b, per_example=K, split=1, T=T, seed=1, dist_id=0, step=0, n=B * K).reshape(B, K)
    for e in range(B):
        base = (e // T) * T
        hi = min(base + T, B)
        assert base <= s[e, 0] < hi                                   # first sample: list a, own tile
        assert np.all((s[e, 1:] >= 1000 + base) & (s[e, 1:] < 1000 + hi))
    # the short last tile (4 examples) is still sampled uniformly over its members
    assert set(s[96:, 0]) <= {96, 97, 98, 99}
    with pytest.raises(ValueError):
        orc.sample_nonconform(a, b, K, 1, T, 1, 0, 0, B * K + 1)


# ---- sample reuse with postponing (Section 4.4) ------------------------------------------------------------------
def test_postponing_worked_examples():
    # nothing local at first: a is postponed (and re-localised), b is postponed, the second a is used, c is
    # postponed, the second b is used; then the postponed ones in the order in which they were postponed
    a, b, c = 5, 9, 2
    assert list(orc.postpone_within_handle([a, b, a, c, b], [])) == [a, b, a, b, c]
    # a local from the start
    assert list(orc.postpone_within_handle([a, b, a, c, b], [a])) == [a, a, b, b, c]
    # a sample that has been postponed is used when it is reached again, even though c never became local before
    assert list(orc.postpone_within_handle([c], [])) == [c]
    assert list(orc.postpone_within_handle([], [1])) == []


def test_postponing_is_a_rearrangement_with_closed_form():
    # every sample is kept (the multiset of the handle is unchanged: what the long-term level needs), samples of
    # local keys keep their order at the front, and exactly the first occurrences of keys that are not local from
    # the start go to the back, in their order
    rng = np.random.default_rng(7)
    for trial in range(30):
        V, n = int(rng.integers(2, 40)), int(rng.integers(0, 200))
        samples = rng.integers(0, V, n)
        resident = rng.choice(V, int(rng.integers(0, V)), replace=False)
        got = orc.postpone_within_handle(samples, resident)
        assert sorted(got) == sorted(samples)
        first = np.zeros(n, dtype=bool)
        seen = set(int(k) for k in resident)
        for i, k in enumerate(samples):
            if int(k) not in seen:
                first[i] = True
                seen.add(int(k))
        assert list(got) == list(samples[~first]) + list(samples[first])
    # everything local: nothing moves; nothing local and all keys distinct: everything is postponed once, in order
    assert list(orc.postpone_within_handle([3, 1, 3, 2], [1, 2, 3])) == [3, 1, 3, 2]
    assert list(orc.postpone_within_handle([4, 2, 7], [])) == [4, 2, 7]


def test_longterm_with_postponing_keeps_the_pool_samples():
    V, P, R = 50, 200, 3
    table = orc.alias_build(np.arange(1, V + 1, dtype=np.float64))
    plain = orc.sample_longterm(table, V, 3, 0, P, R, 40, 300)
    post = orc.sample_longterm_postponed(table, V, 3, 0, P, R, 40, 300, resident_keys=[49, 48, 47])
    assert sorted(post) == sorted(plain) and not np.array_equal(post, plain)
    assert np.array_equal(orc.sample_longterm_postponed(table, V, 3, 0, P, R, 40, 300, range(V)), plain)
