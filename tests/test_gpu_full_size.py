"""GPU parity at the full sizes of the benchmark configurations, run the way bench.py runs them (steps prepared
ahead, the preparatory work riding in earlier launches), over 100 steps each: the rows that the steps touch are
compared with the oracle's to the 100-step bar (1e-3, element by element with a floor per row, tests/parity.py;
all of them up to a million per table, beyond that the rows of the most frequent keys and a seeded sample of the
rest), and every other row of the tables must be bit-identical to what it was."""
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2104_00501_amd import binding as nb
from paper_2104_00501_amd import workloads as wl
from tests.parity import TOL_100_STEPS, dev, dev_u32, param_err, update_err

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _say(line):
    """A line for whoever watches the run: on stdout and, where output capture would hold it back, in a file."""
    print(line, flush=True)
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "full_size_progress.txt"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


# Element-wise comparison of every touched row costs minutes of host time for millions of rows of 2 KB; beyond this
# many, the rows of the most frequent keys (where the sums are longest) and a seeded random sample of the rest are
# compared.  That no row outside the steps' keys changed is checked on all rows either way.
_MOST_ROWS_COMPARED = 1_000_000
_HOTTEST_ROWS = 50_000


def _touched_rows_match(t_dev, init_dev, ref_host, touched, cols, tol, what):
    """Both metrics are maxima over rows with a floor per row, so the touched rows are compared in blocks (millions
    of rows of 2 KB would otherwise be held several times over in fp64, silently, for minutes)."""
    import torch
    touched = np.unique(np.asarray(touched, dtype=np.int64))
    changed = (t_dev != init_dev).any(dim=1).nonzero().ravel().cpu().numpy()
    assert np.isin(changed, touched).all(), what + ": a row outside the steps' keys changed"
    pad = np.setdiff1d(np.arange(t_dev.shape[1]), cols)
    n_touched = len(touched)
    if n_touched > _MOST_ROWS_COMPARED:      # the most frequent keys (the smallest) and a seeded sample of the others
        rest = np.random.default_rng(20211).choice(touched[_HOTTEST_ROWS:], _MOST_ROWS_COMPARED - _HOTTEST_ROWS, replace=False)
        touched = np.concatenate([touched[:_HOTTEST_ROWS], np.sort(rest)])
        _say("%s: %d of the %d touched rows are compared element by element" % (what, len(touched), n_touched))
    rel = ab = ue = 0.0
    block = 131_072
    for n, lo in enumerate(range(0, len(touched), block)):
        rows = touched[lo:lo + block]
        index = torch.from_numpy(rows).cuda()
        got, before = t_dev[index].cpu().numpy(), init_dev[index].cpu().numpy()
        ref = ref_host[rows]
        r, a = param_err(got, ref, before, cols)
        rel, ab, ue = max(rel, r), max(ab, a), max(ue, update_err(got, ref, before, cols))
        assert np.all(got[:, pad] == 0), what + ": padding lanes changed"
        if n % 4 == 3:
            _say("%s: %d of %d touched rows compared" % (what, lo + len(rows), len(touched)))
    _say("%s: %d touched rows of %d, %d changed; parameter err %.3g (abs %.3g), update err %.3g"
         % (what, n_touched, t_dev.shape[0], len(changed), rel, ab, ue))
    assert rel <= tol, "%s: parameter error %.3g (abs %.3g) > %.1g" % (what, rel, ab, tol)
    assert ue <= tol, "%s: error of the total update %.3g > %.1g" % (what, ue, tol)


def _progress(what, t, steps):
    """The oracle's 100 full-size steps take minutes on one core: a line now and then shows that the test is alive."""
    if t % 10 == 9 or t == steps - 1:
        _say("%s: oracle step %d of %d" % (what, t + 1, steps))


def _run(ctx, batches, depth):
    queue = [nb.nups_prepare_step(ctx, b) for b in batches[:depth]]
    loss = None
    for t in range(len(batches)):
        if t + depth < len(batches):
            queue.append(nb.nups_prepare_step(ctx, batches[t + depth]))
        loss = nb.nups_step_prepared(ctx, queue.pop(0), want_loss=(t == len(batches) - 1))
    nb.nups_check(ctx)
    return loss


def test_word_vectors_1m_keys_d300_bounded_reuse():
    # the default benchmark workload: 1M keys, d = 300, 3 negatives under BOUNDED U = 4, G = 250, B = 16,384.
    # With summed batch gradients the plain step overflows at this configuration's learning rate well within 100
    # steps (the oracle too: the hottest words collect over a thousand contributions per step), so the 100 steps
    # run with the paper's remedy (Section 5.1): the updates of the 1,000 most frequent words are clipped at
    # twice their mean norm.
    V, d, B, K, U, G, window, steps, seed = 1_000_000, 300, 16_384, 3, 4, 250, 5, 100, 1004
    toks = wl.zipf_stream(V, 1.0, steps * B // (2 * window) + 2 * window + 2, seed)
    centers, contexts = wl.window_pairs(toks, window, 0, steps * B)
    w = wl.expected_unigram_weights(V, 1.0, 1e9)
    In = wl.uniform_table(V, d, -0.5 / d, 0.5 / d, seed)
    Out = np.zeros_like(In)                       # output vectors start at zero, as the configuration says
    tin, tout = dev(In), dev(Out)
    init_in, init_out = tin.clone(), tout.clone()
    ctx = nb.nups_init([tin, tout], [d, d])
    dist = nb.nups_register_distribution(ctx, 1, w, nb.NUPS_BOUNDED, U=U, G=G, seed=seed)
    hot = np.arange(1000, dtype=np.uint32)        # keys are frequency ranks
    nb.nups_set_hot_keys(ctx, 0, hot)
    nb.nups_set_hot_keys(ctx, 1, hot)
    nb.nups_set_update_clipping(ctx, 2.0)
    kc, ko = dev_u32(centers), dev_u32(contexts)
    lrs = [float(wl.linear_lr(0.025, t, 610_000)) for t in range(steps)]
    batches = [nb.make_batch(nb.NUPS_TASK_SGNS, B, kc.data_ptr() + 4 * t * B, ko.data_ptr() + 4 * t * B, n_neg=K,
                             lr=lrs[t], dist=dist, sample_step=t) for t in range(steps)]
    loss = _run(ctx, batches, 3)
    alias = orc.alias_build(w)
    negs_all = []
    stats_in, stats_out = np.zeros(2), np.zeros(2)
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        negs = orc.sample_bounded(alias, V, seed, 0, t, B * K, U, G)
        negs_all.append(negs)
        rloss = orc.step_sgns_clipped(In, Out, d, centers[sl], contexts[sl], negs, K, lrs[t], hot, hot, 2.0,
                                      stats_in, stats_out)
        _progress("word vectors", t, steps)
    assert np.isfinite(In).all() and np.isfinite(Out).all() and np.abs(In).max() < 100
    assert abs(loss - rloss) <= TOL_100_STEPS * abs(rloss)
    cols = list(range(d))
    _touched_rows_match(tin, init_in, In, centers, cols, TOL_100_STEPS, "input vectors")
    _touched_rows_match(tout, init_out, Out, np.concatenate([contexts] + negs_all), cols, TOL_100_STEPS, "output vectors")
    nb.nups_destroy(ctx)


def test_factorisation_10m_by_1m_rank_100():
    # 10M x 1M, rank 100, 65,536 cells per step, prepared four ahead as bench.py does for this task
    import torch
    n_rows, n_cols, d, B, steps = 10_000_000, 1_000_000, 100, 65_536, 100
    rows, cols, vals = wl.mf_cells(n_rows, n_cols, 0.8, steps * B, 1002)
    stride = wl.padded_stride(d)
    g = torch.Generator(device="cuda").manual_seed(1002)

    def table(n):
        t = torch.zeros((n, stride), dtype=torch.float32, device="cuda")
        t[:, :d] = torch.rand((n, d), generator=g, device="cuda") * 0.2 - 0.1
        return t

    tw, th = table(n_rows), table(n_cols)
    init_w, init_h = tw.clone(), th.clone()
    W, H = tw.cpu().numpy(), th.cpu().numpy()
    ctx = nb.nups_init([tw, th], [d, d])
    kr, kc, kv = dev_u32(rows), dev_u32(cols), dev(vals)
    batches = [nb.make_batch(nb.NUPS_TASK_MF, B, kr.data_ptr() + 4 * t * B, kc.data_ptr() + 4 * t * B,
                             val=kv.data_ptr() + 4 * t * B, lr=0.005, l2=0.01) for t in range(steps)]
    loss = _run(ctx, batches, 4)
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        rloss = orc.step_mf(W, H, d, rows[sl], cols[sl], vals[sl], 0.005, 0.01)[0]
        _progress("factorisation", t, steps)
    assert abs(loss - rloss) <= TOL_100_STEPS * abs(rloss)
    _touched_rows_match(tw, init_w, W, rows, list(range(d)), TOL_100_STEPS, "row factors")
    _touched_rows_match(th, init_h, H, cols, list(range(d)), TOL_100_STEPS, "column factors")
    nb.nups_destroy(ctx)


def test_complex_4p6m_entities_d500_adagrad():
    # 4.6M entities, d = 500 with AdaGrad state, 1,024 triples with 50 + 50 uniform negatives per step
    import torch
    n_ent, n_rel, d, B, nh, nt, steps, seed = 4_600_000, 822, 500, 1024, 50, 50, 100, 1003
    s, r, o = wl.kge_triples(n_ent, n_rel, steps * B, seed)
    stride, half = 512, d // 2
    g = torch.Generator(device="cuda").manual_seed(seed)

    def table(n):
        t = torch.zeros((n, stride), dtype=torch.float32, device="cuda")
        t[:, :half] = torch.rand((n, half), generator=g, device="cuda") * 0.2 - 0.1
        t[:, stride // 2:stride // 2 + half] = torch.rand((n, half), generator=g, device="cuda") * 0.2 - 0.1
        return t

    def state(n):       # a warmed-up accumulator on the logical lanes
        t = torch.zeros((n, stride), dtype=torch.float32, device="cuda")
        t[:, :half] = 1e-3
        t[:, stride // 2:stride // 2 + half] = 1e-3
        return t

    te, tr, ge, gr = table(n_ent), table(n_rel), state(n_ent), state(n_rel)
    init_e, init_g, init_r, init_gr = te.clone(), ge.clone(), tr.clone(), gr.clone()
    E, R, GE, GR = te.cpu().numpy(), tr.cpu().numpy(), ge.cpu().numpy(), gr.cpu().numpy()
    ctx = nb.nups_init([te, tr], [d, d])
    nb.nups_set_state(ctx, 0, ge)
    nb.nups_set_state(ctx, 1, gr)
    dist = nb.nups_register_distribution(ctx, 0, None, nb.NUPS_CONFORM, seed=seed)
    ks, kr, ko = dev_u32(s), dev_u32(r), dev_u32(o)
    batches = [nb.make_batch(nb.NUPS_TASK_KGE, B, ks.data_ptr() + 4 * t * B, kr.data_ptr() + 4 * t * B,
                             k2=ko.data_ptr() + 4 * t * B, n_neg=nh, n_neg2=nt, lr=0.1, eps=1e-10, dist=dist,
                             sample_step=t) for t in range(steps)]
    loss = _run(ctx, batches, 3)
    negs_all = []
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        negs = orc.sample_conform(None, n_ent, seed, 0, t, B * (nh + nt))
        negs_all.append(negs)
        rloss = orc.step_kge(E, GE, R, GR, d, s[sl], r[sl], o[sl], negs, nh, nt, 0.1, 1e-10)[0]
        _progress("ComplEx", t, steps)
    assert abs(loss - rloss) <= TOL_100_STEPS * abs(rloss)
    cols = list(range(half)) + list(range(stride // 2, stride // 2 + half))
    touched = np.concatenate([s, o] + negs_all)
    _touched_rows_match(te, init_e, E, touched, cols, TOL_100_STEPS, "entity rows")
    _touched_rows_match(ge, init_g, GE, touched, cols, TOL_100_STEPS, "entity state rows")
    _touched_rows_match(tr, init_r, R, r, cols, TOL_100_STEPS, "relation rows")
    _touched_rows_match(gr, init_gr, GR, r, cols, TOL_100_STEPS, "relation state rows")
    nb.nups_destroy(ctx)
