"""Pins for the oracle's norm clipping of hot-key updates (Section 5.1: updates of replicated parameters that
exceed the average norm by more than a factor are clipped): a two-step example worked by hand, reduction to the
plain step, invariants that hold for any input, and the purpose the paper states for it (CPU only)."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2104_00501_amd import workloads as wl


def _stats():
    return np.zeros(2, dtype=np.float64)


def _table(rows, stride=64):
    t = np.zeros((len(rows), stride), dtype=np.float32)
    for i, r in enumerate(rows):
        t[i, :len(r)] = r
    return t


def test_two_factorisation_steps_worked_by_hand():
    # One row (hot), two columns (not hot), rank 2, no regulariser, lr = 1/8.  All numbers are dyadic, so every
    # value below is exact in binary floating point and the expected tables can be written down.
    W = _table([[1.0, 0.0]])
    H = _table([[0.5, 0.5], [0.0, 2.0]])
    lr, sw, sh = 0.125, _stats(), _stats()
    # step 1: cell (0, 0) = 1: error 1 - 0.5 = 0.5; dW = -2 * 0.5 * H0 = (-0.5, -0.5), norm sqrt(0.5);
    # dH0 = -2 * 0.5 * W0 = (-1, 0).  Nothing has been seen yet, so nothing is clipped.
    orc.step_mf_clipped(W, H, 2, [0], [0], np.float32([1.0]), lr, 0.0, [0], [], 2.0, sw, sh)
    assert np.array_equal(W[0, :2], np.float32([1.0625, 0.0625]))
    assert np.array_equal(H[0, :2], np.float32([0.625, 0.5]))
    assert sw[1] == 1.0 and abs(sw[0] - np.sqrt(0.5)) < 1e-15
    assert np.array_equal(sh, [0.0, 0.0])                       # column 0 is not hot: not measured
    # step 2: cell (0, 1) = 8.125: error 8.125 - 2 * 0.0625 = 8; dW = -16 * H1 = (0, -32), norm 32, more than
    # the bound 2 * sqrt(0.5) = sqrt(2): clipped to (0, -sqrt(2)).  dH1 = -16 * W0 = (-17, -1): not hot, unclipped.
    orc.step_mf_clipped(W, H, 2, [0], [1], np.float32([8.125]), lr, 0.0, [0], [], 2.0, sw, sh)
    assert W[0, 0] == np.float32(1.0625)
    assert W[0, 1] == np.float32(0.0625 + lr * np.sqrt(2.0))
    assert np.array_equal(H[1, :2], np.float32([0.0 + lr * 17.0, 2.0 + lr * 1.0]))
    assert sw[1] == 2.0 and abs(sw[0] - (np.sqrt(0.5) + 32.0)) < 1e-13       # the norm before clipping is recorded
    # step 3: the mean is now (sqrt(0.5) + 32) / 2, the bound sqrt(0.5) + 32 = 32.7...; the same cell's update
    # (norm 32.2) passes unchanged.
    w, h = np.float64(W[0, :2]), np.float64(H[1, :2])
    err = 8.125 - (w[0] * h[0] + w[1] * h[1])
    assert 32.0 < 2.0 * err * np.linalg.norm(h) < np.sqrt(0.5) + 32.0
    orc.step_mf_clipped(W, H, 2, [0], [1], np.float32([8.125]), lr, 0.0, [0], [], 2.0, sw, sh)
    assert np.array_equal(W[0, :2], np.float32(w + lr * 2.0 * err * h))
    assert sw[1] == 3.0


def _sgns_case(seed, V=40, d=5, B=300, K=3, stride=64):
    rng = np.random.default_rng(seed)
    In = np.zeros((V, stride), dtype=np.float32)
    Out = np.zeros((V, stride), dtype=np.float32)
    In[:, :d] = rng.uniform(-1, 1, (V, d))
    Out[:, :d] = rng.uniform(-1, 1, (V, d))
    p = wl.zipf_pmf(V, 1.0)
    c = rng.choice(V, B, p=p).astype(np.uint32)
    o = rng.choice(V, B, p=p).astype(np.uint32)
    ng = rng.choice(V, B * K, p=p).astype(np.uint32)
    return In, Out, c, o, ng


def test_no_hot_keys_or_an_unreachable_bound_is_the_plain_step():
    d, K, lr = 5, 3, 0.05
    In, Out, c, o, ng = _sgns_case(1)
    ref_in, ref_out = In.copy(), Out.copy()
    ref_loss = orc.step_sgns(ref_in, ref_out, d, c, o, ng, K, lr)[0]
    a_in, a_out, si, so = In.copy(), Out.copy(), _stats(), _stats()
    loss = orc.step_sgns_clipped(a_in, a_out, d, c, o, ng, K, lr, [], None, 2.0, si, so)
    assert loss == ref_loss and np.array_equal(a_in, ref_in) and np.array_equal(a_out, ref_out)
    assert not si.any() and not so.any()
    b_in, b_out = In.copy(), Out.copy()
    si[:] = (3.0, 2.0)
    so[:] = (1.0, 4.0)
    orc.step_sgns_clipped(b_in, b_out, d, c, o, ng, K, lr, np.arange(10), np.arange(10), 1e30, si, so)
    assert np.array_equal(b_in, ref_in) and np.array_equal(b_out, ref_out)
    assert si[1] == 2.0 + len(np.intersect1d(c, np.arange(10)))            # still measured
    assert so[1] == 4.0 + len(np.intersect1d(np.concatenate([o, ng]), np.arange(10)))


@pytest.mark.parametrize("seed,factor", [(2, 2.0), (3, 0.5), (4, 1.0)])
def test_clipped_updates_are_shortened_not_turned_and_everything_else_is_untouched(seed, factor):
    d, K, lr = 5, 3, 0.05
    In, Out, c, o, ng = _sgns_case(seed)
    hot_in, hot_out = np.arange(8), np.arange(12)
    # the plain step gives every key's summed gradient: (before - after) / lr
    p_in, p_out = In.copy(), Out.copy()
    orc.step_sgns(p_in, p_out, d, c, o, ng, K, lr)
    si, so = np.float64([0.9, 3.0]), np.float64([2.0, 5.0])               # means 0.3 and 0.4 from earlier steps
    bounds = factor * si[0] / si[1], factor * so[0] / so[1]
    c_in, c_out = In.copy(), Out.copy()
    orc.step_sgns_clipped(c_in, c_out, d, c, o, ng, K, lr, hot_in, hot_out, factor, si, so)
    n_clipped = 0
    for before, plain, clipped, hot, bound, stats, start, touched in (
            (In, p_in, c_in, hot_in, bounds[0], si, (0.9, 3.0), np.unique(c)),
            (Out, p_out, c_out, hot_out, bounds[1], so, (2.0, 5.0), np.unique(np.concatenate([o, ng])))):
        full = (np.float64(before) - np.float64(plain)) / lr
        got = (np.float64(before) - np.float64(clipped)) / lr
        cold = np.setdiff1d(np.arange(len(before)), hot)
        assert np.array_equal(clipped[cold], plain[cold])                  # keys outside the hot set: bit-identical
        norms = np.linalg.norm(full[hot], axis=1)
        for k, n in zip(hot, norms):
            if n <= bound * (1 - 1e-6):
                assert np.allclose(got[k], full[k], rtol=0, atol=2e-6)     # short enough: passes unchanged
            elif n >= bound * (1 + 1e-6):
                n_clipped += 1
                assert abs(np.linalg.norm(got[k]) - bound) < 3e-6          # as long as the bound allows
                assert np.allclose(got[k] / bound, full[k] / n, rtol=0, atol=1e-5)   # same direction
        hot_touched = np.intersect1d(hot, touched)
        assert stats[1] == start[1] + len(hot_touched)
        assert abs(stats[0] - start[0] - norms[np.isin(hot, hot_touched)].sum()) < 1e-5   # norms before clipping
    assert n_clipped >= 3                                                  # the case exercises the clipping


def test_a_step_is_clipped_against_earlier_steps_only_and_in_any_order():
    d, K, lr = 5, 3, 0.05
    In, Out, c, o, ng = _sgns_case(5)
    hot = np.arange(10)
    a_in, a_out, si, so = In.copy(), Out.copy(), np.float64([0.5, 2.0]), np.float64([0.5, 2.0])
    orc.step_sgns_clipped(a_in, a_out, d, c, o, ng, K, lr, hot, hot, 2.0, si, so)
    # the same examples in another order (each with its own negatives): same result up to fp64 rounding of sums
    perm = np.random.default_rng(0).permutation(len(c))
    b_in, b_out, ti, to = In.copy(), Out.copy(), np.float64([0.5, 2.0]), np.float64([0.5, 2.0])
    orc.step_sgns_clipped(b_in, b_out, d, c[perm], o[perm], ng.reshape(-1, K)[perm].ravel(), K, lr, hot, hot, 2.0, ti, to)
    assert np.max(np.abs(a_in - b_in)) < 1e-6 and np.max(np.abs(a_out - b_out)) < 1e-6
    assert abs(si[0] - ti[0]) < 1e-9 and si[1] == ti[1]
    # the keys' own numbering plays no part either: with the tables' rows and all keys reversed, same result
    V = len(In)
    r_in, r_out, ri, ro = In[::-1].copy(), Out[::-1].copy(), np.float64([0.5, 2.0]), np.float64([0.5, 2.0])
    orc.step_sgns_clipped(r_in, r_out, d, V - 1 - c, V - 1 - o, V - 1 - ng, K, lr, V - 1 - hot, V - 1 - hot, 2.0, ri, ro)
    assert np.max(np.abs(a_in - r_in[::-1])) < 1e-6 and np.max(np.abs(a_out - r_out[::-1])) < 1e-6


def test_clipping_keeps_the_small_word_vector_configuration_finite():
    # Summed gradients at lr = 0.025 blow the plain step up within 100 steps of the small configuration (the
    # hottest word collects some 400 contributions per step); the paper clips for that reason.
    V, d, B, K, window, steps, lr = 10_000, 100, 4096, 5, 2, 100, 0.025
    toks = wl.zipf_stream(V, 1.0, steps * B // (2 * window) + 2 * window + 2, 1001)
    centers, contexts = wl.window_pairs(toks, window, 0, steps * B)
    weights = wl.unigram_weights(toks, V)
    alias = orc.alias_build(weights)
    hot = np.arange(100)                     # keys are frequency ranks
    plain, clipped = wl.sgns_tables(V, d, 1001), wl.sgns_tables(V, d, 1001)
    si, so = _stats(), _stats()
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        ng = orc.sample_conform(alias, V, 1001, 0, t, B * K)
        with np.errstate(all="ignore"):
            orc.step_sgns(plain[0], plain[1], d, centers[sl], contexts[sl], ng, K, lr)
        orc.step_sgns_clipped(clipped[0], clipped[1], d, centers[sl], contexts[sl], ng, K, lr, hot, hot, 2.0, si, so)
    assert not np.isfinite(plain[0]).all() or np.abs(plain[0]).max() > 1e6
    assert np.isfinite(clipped[0]).all() and np.isfinite(clipped[1]).all()
    assert max(np.abs(clipped[0]).max(), np.abs(clipped[1]).max()) < 50.0
