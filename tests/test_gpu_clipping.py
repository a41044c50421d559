"""GPU parity of the steps with norm clipping of hot-key updates (Section 5.1) against the CPU oracle: the
recorded norm statistics (count exact, sum to rounding) and the tables, to the bars of the plain steps."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2104_00501_amd import binding as nb
from paper_2104_00501_amd import workloads as wl
from tests.parity import assert_table, dev, dev_u32

pytestmark = pytest.mark.gpu


def _close(got, ref, before, d, tol, what):
    assert_table(got, ref, before, list(range(d)), tol, what, tol_update=tol)


def _stats_match(ctx, table, ref, what):
    norm_sum, count = nb.nups_get_update_clipping(ctx, table)
    print("%s: %d norms, sum %.9g (oracle %.9g)" % (what, count, norm_sum, ref[0]))
    assert count == ref[1], what
    assert abs(norm_sum - ref[0]) <= 1e-5 * max(ref[0], 1e-30), what


def _sgns_run(V, d, B, K, window, lr, steps, hot, factor, depth, seed, declare=True):
    toks = wl.zipf_stream(V, 1.0, steps * B // (2 * window) + 2 * window + 2, seed)
    centers, contexts = wl.window_pairs(toks, window, 0, steps * B)
    w = wl.unigram_weights(toks, V)
    In, Out = wl.sgns_tables(V, d, seed)
    Out[:] = wl.uniform_table(V, d, -0.5 / d, 0.5 / d, seed + 1)
    tin, tout = dev(In), dev(Out)
    ctx = nb.nups_init([tin, tout], [d, d])
    dist = nb.nups_register_distribution(ctx, 1, w, nb.NUPS_CONFORM, seed=seed)
    hot_keys = np.arange(hot, dtype=np.uint32)
    if declare:
        nb.nups_set_hot_keys(ctx, 0, hot_keys)
        nb.nups_set_hot_keys(ctx, 1, hot_keys)
    nb.nups_set_update_clipping(ctx, factor)
    kc, ko = dev_u32(centers), dev_u32(contexts)
    batches = [nb.make_batch(nb.NUPS_TASK_SGNS, B, kc.data_ptr() + 4 * t * B, ko.data_ptr() + 4 * t * B, n_neg=K,
                             lr=lr, dist=dist, sample_step=t) for t in range(steps)]
    queue = [nb.nups_prepare_step(ctx, b) for b in batches[:depth]]
    for t in range(steps):
        if depth and t + depth < steps:
            queue.append(nb.nups_prepare_step(ctx, batches[t + depth]))
        if depth:
            nb.nups_step_prepared(ctx, queue.pop(0))
        else:
            nb.nups_step(ctx, batches[t])
    nb.nups_check(ctx)
    alias = orc.alias_build(w)
    rin, rout, si, so = In.copy(), Out.copy(), np.zeros(2), np.zeros(2)
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        negs = orc.sample_conform(alias, V, seed, 0, t, B * K)
        orc.step_sgns_clipped(rin, rout, d, centers[sl], contexts[sl], negs, K, lr, hot_keys if declare else [],
                              hot_keys if declare else [], factor, si, so)
    return ctx, tin.cpu().numpy(), tout.cpu().numpy(), rin, rout, si, so, In, Out


@pytest.mark.parametrize("steps,depth,tol", [(2, 0, 2e-5), (30, 3, 1e-3)])
def test_sgns_steps_with_clipping(steps, depth, tol):
    # the small word-vector configuration at the learning rate at which the plain step diverges; the 100 most
    # frequent words are hot: the hottest take the chunked path, the others single row groups
    V, d, B, K = 10_000, 100, 4096, 5
    ctx, gin, gout, rin, rout, si, so, In, Out = _sgns_run(V, d, B, K, 2, 0.025, steps, 100, 2.0, depth, 1001)
    assert si[1] > 50 * steps and so[1] > 50 * steps
    _stats_match(ctx, 0, si, "input table")
    _stats_match(ctx, 1, so, "output table")
    _close(gin, rin, In, d, tol, "input table after %d clipped steps" % steps)
    _close(gout, rout, Out, d, tol, "output table after %d clipped steps" % steps)
    nb.nups_destroy(ctx)


def test_sgns_clipping_really_clips_and_wide_rows():
    # a tight factor, so that most hot-key updates are shortened, on 300-float rows
    V, d, B, K = 3_000, 300, 1500, 3
    ctx, gin, gout, rin, rout, si, so, In, Out = _sgns_run(V, d, B, K, 5, 0.01, 6, 40, 0.5, 1, 77)
    _stats_match(ctx, 0, si, "input table")
    _stats_match(ctx, 1, so, "output table")
    _close(gin, rin, In, d, 1e-4, "input table")
    _close(gout, rout, Out, d, 1e-4, "output table")
    nb.nups_destroy(ctx)


def test_clipping_without_a_declared_hot_set_measures_and_changes_nothing():
    V, d, B, K = 2_000, 64, 1024, 2
    ctx, gin, gout, rin, rout, si, so, In, Out = _sgns_run(V, d, B, K, 2, 0.01, 3, 0, 2.0, 1, 5, declare=False)
    assert nb.nups_get_update_clipping(ctx, 0) == (0.0, 0.0) and nb.nups_get_update_clipping(ctx, 1) == (0.0, 0.0)
    assert not si.any() and not so.any()
    _close(gin, rin, In, d, 1e-4, "input table")
    _close(gout, rout, Out, d, 1e-4, "output table")
    nb.nups_destroy(ctx)


def test_mf_steps_with_clipping():
    n_rows, n_cols, d, B, steps, lr, l2 = 5_000, 2_000, 100, 8192, 6, 0.005, 0.01
    rows, cols, vals = wl.mf_cells(n_rows, n_cols, 1.1, steps * B, 9)
    W, H = wl.uniform_table(n_rows, d, -0.1, 0.1, 10), wl.uniform_table(n_cols, d, -0.1, 0.1, 11)
    tw, th = dev(W), dev(H)
    ctx = nb.nups_init([tw, th], [d, d])
    hot_w, hot_h = np.arange(60, dtype=np.uint32), np.arange(30, dtype=np.uint32)
    nb.nups_set_hot_keys(ctx, 0, hot_w)
    nb.nups_set_hot_keys(ctx, 1, hot_h)
    with pytest.raises(nb.NupsError) as e:
        nb.nups_get_update_clipping(ctx, 0)
    assert e.value.status == nb.NUPS_ERR_STATE
    with pytest.raises(nb.NupsError) as e:
        nb.nups_set_update_clipping(ctx, -1.0)
    assert e.value.status == nb.NUPS_ERR_ARG
    nb.nups_set_update_clipping(ctx, 2.0)
    kr, kc = dev_u32(rows), dev_u32(cols)
    import torch
    kv = torch.from_numpy(vals).cuda()
    rw, rh, sw, sh = W.copy(), H.copy(), np.zeros(2), np.zeros(2)
    for t in range(steps):
        if t == 4:
            nb.nups_set_update_clipping(ctx, 0.0)        # off: the step is the plain one and records nothing
        if t == 5:
            nb.nups_set_update_clipping(ctx, 1.0)        # on again: statistics start afresh
            sw[:] = 0.0
            sh[:] = 0.0
        nb.nups_step(ctx, nb.make_batch(nb.NUPS_TASK_MF, B, kr.data_ptr() + 4 * t * B, kc.data_ptr() + 4 * t * B,
                                        val=kv.data_ptr() + 4 * t * B, lr=lr, l2=l2))
        sl = slice(t * B, (t + 1) * B)
        if t == 4:
            orc.step_mf(rw, rh, d, rows[sl], cols[sl], vals[sl], lr, l2)
        else:
            orc.step_mf_clipped(rw, rh, d, rows[sl], cols[sl], vals[sl], lr, l2, hot_w, hot_h, 2.0 if t < 4 else 1.0,
                                sw, sh)
        if t == 3:
            _stats_match(ctx, 0, sw, "row factors after four steps")
            _stats_match(ctx, 1, sh, "column factors after four steps")
    nb.nups_check(ctx)
    _stats_match(ctx, 0, sw, "row factors")
    _stats_match(ctx, 1, sh, "column factors")
    _close(tw.cpu().numpy(), rw, W, d, 1e-4, "row factors")
    _close(th.cpu().numpy(), rh, H, d, 1e-4, "column factors")
    nb.nups_destroy(ctx)
