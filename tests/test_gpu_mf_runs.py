"""GPU parity of the factorisation step where the cells of a batch stand in the visiting order of the paper's workers
(Section 5.1: column by column) and the rows are wide enough (256 floats and more) for the gradient kernel to add up
the column gradients of runs of cells with one column: single steps, steps prepared ahead, deterministic mode, norm
clipping and stale replicas, each against the oracle (which knows nothing of runs: it sums every key's contributions in
fp64)."""
import numpy as np
import pytest

from oracle import oracle as orc
from oracle import replicas as rep
from paper_2104_00501_amd import binding as nb
from paper_2104_00501_amd import workloads as wl
from tests.parity import TOL_ONE_STEP, TOL_UPDATE, assert_table, dev, dev_u32
from tests.test_gpu_replicas import _extended
from tests.test_gpu_steps import _assert_structure

pytestmark = pytest.mark.gpu


def _cells_by_column(nr, nc, s, B, steps, seed):
    rows, cols, vals = wl.mf_cells(nr, nc, s, B * steps * 8, seed)
    rows, cols, vals = wl.mf_visit_by_column(rows, cols, vals, B, seed + 1)
    assert len(rows) >= B * steps
    return rows[:B * steps].copy(), cols[:B * steps].copy(), vals[:B * steps].copy()


def _runs(cols):
    """Lengths of the runs of equal columns inside blocks of 16 consecutive cells (what the gradient kernel sees)."""
    head = np.ones(len(cols), dtype=bool)
    head[1:] = cols[1:] != cols[:-1]
    head[::16] = True
    return np.diff(np.append(np.flatnonzero(head), len(cols)))


@pytest.mark.parametrize("nr,nc,d,B,s", [
    (20_000, 2_000, 250, 8_192, 1.1),      # rows of 256 floats, the narrowest that take this path
    (6_000, 800, 1000, 4_096, 1.1),        # the paper's rank (Table 1): rows of 1,024 floats
    (3_000, 50, 300, 1_024, 0.6),          # few columns: every worker's cells are long runs of one column
    (500, 300, 500, 64, 1.1),              # one cell per worker: no run longer than a cell or two
])
def test_one_step_by_column_matches_the_oracle(nr, nc, d, B, s):
    rows, cols, vals = _cells_by_column(nr, nc, s, B, 1, 31)
    if B >= 1024:
        assert _runs(cols).max() == 16 and np.bincount(cols).max() > 16      # whole blocks of one column, hot columns
        counts = np.bincount(cols, minlength=nc)
        assert ((counts > 1) & (counts <= 16)).any()                           # and columns that may sit in one run
    W, H = wl.uniform_table(nr, d, -0.1, 0.1, 1), wl.uniform_table(nc, d, -0.1, 0.1, 2)
    tw, th = dev(W), dev(H)
    ctx = nb.nups_init([tw, th], [d, d])
    batch = nb.make_batch(nb.NUPS_TASK_MF, B, dev_u32(rows), dev_u32(cols), val=dev(vals), lr=0.005, l2=0.01)
    keep = (batch,)
    loss = nb.nups_step(ctx, batch, want_loss=True)
    rw, rh = W.copy(), H.copy()
    rloss, sw, sh = orc.step_mf(rw, rh, d, rows, cols, vals, 0.005, 0.01)
    _assert_structure(ctx, 0, B, sw)
    _assert_structure(ctx, 1, B, sh)
    assert_table(tw.cpu().numpy(), rw, W, list(range(d)), TOL_ONE_STEP, "row factors", tol_update=TOL_UPDATE)
    assert_table(th.cpu().numpy(), rh, H, list(range(d)), TOL_ONE_STEP, "column factors", tol_update=TOL_UPDATE)
    assert abs(loss - rloss) <= 1e-5 * abs(rloss)
    del keep
    nb.nups_destroy(ctx)


def _run_steps(ctx, kr, kc, kv, B, steps, depth):
    batches = [nb.make_batch(nb.NUPS_TASK_MF, B, kr.data_ptr() + 4 * t * B, kc.data_ptr() + 4 * t * B,
                             val=kv.data_ptr() + 4 * t * B, lr=0.005, l2=0.01) for t in range(steps)]
    queue = [nb.nups_prepare_step(ctx, b) for b in batches[:depth]]
    for t in range(steps):
        if t + depth < steps:
            queue.append(nb.nups_prepare_step(ctx, batches[t + depth]))
        if depth:
            nb.nups_step_prepared(ctx, queue.pop(0))
        else:
            nb.nups_step(ctx, batches[t])
    nb.nups_check(ctx)


@pytest.mark.parametrize("depth,deterministic,hot", [(4, False, None), (3, True, None), (0, True, 0), (4, True, 40)])
def test_steps_by_column_prepared_ahead_and_in_deterministic_mode(depth, deterministic, hot):
    nr, nc, d, B, steps = 20_000, 1_500, 250, 4_096, 6
    rows, cols, vals = _cells_by_column(nr, nc, 1.1, B, steps, 41)
    W, H = wl.uniform_table(nr, d, -0.1, 0.1, 3), wl.uniform_table(nc, d, -0.1, 0.1, 4)
    kr, kc, kv = dev_u32(rows), dev_u32(cols), dev(vals)
    tables = []
    for _ in range(2 if deterministic else 1):
        tw, th = dev(W), dev(H)
        ctx = nb.nups_init([tw, th], [d, d])
        if deterministic:
            nb.nups_set_deterministic(ctx, 1)
        if hot is not None:                     # an empty set switches the chunked path off, a set declares it
            for table in (0, 1):
                nb.nups_set_hot_keys(ctx, table, np.arange(hot, dtype=np.uint32))
        _run_steps(ctx, kr, kc, kv, B, steps, depth)
        tables.append((tw.cpu().numpy(), th.cpu().numpy()))
        nb.nups_destroy(ctx)
    rw, rh = W.copy(), H.copy()
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        orc.step_mf(rw, rh, d, rows[sl], cols[sl], vals[sl], 0.005, 0.01)
    assert_table(tables[0][0], rw, W, list(range(d)), 1e-4, "row factors", tol_update=1e-4)
    assert_table(tables[0][1], rh, H, list(range(d)), 1e-4, "column factors", tol_update=1e-4)
    if deterministic:
        assert np.array_equal(tables[0][0], tables[1][0]) and np.array_equal(tables[0][1], tables[1][1]), \
            "two runs in deterministic mode differ"


def test_deterministic_results_do_not_depend_on_the_hot_set():
    nr, nc, d, B, steps = 8_000, 600, 250, 4_096, 3
    rows, cols, vals = _cells_by_column(nr, nc, 1.1, B, steps, 43)
    W, H = wl.uniform_table(nr, d, -0.1, 0.1, 5), wl.uniform_table(nc, d, -0.1, 0.1, 6)
    kr, kc, kv = dev_u32(rows), dev_u32(cols), dev(vals)
    results = []
    for hot in (None, 0, 25):
        tw, th = dev(W), dev(H)
        ctx = nb.nups_init([tw, th], [d, d])
        nb.nups_set_deterministic(ctx, 1)
        if hot is not None:
            for table in (0, 1):
                nb.nups_set_hot_keys(ctx, table, np.arange(hot, dtype=np.uint32))
        _run_steps(ctx, kr, kc, kv, B, steps, 4)
        results.append((tw.cpu().numpy(), th.cpu().numpy()))
        nb.nups_destroy(ctx)
    for w, h in results[1:]:
        assert np.array_equal(w, results[0][0]) and np.array_equal(h, results[0][1])


def test_steps_by_column_with_clipping():
    nr, nc, d, B, steps, lr, l2 = 6_000, 900, 250, 4_096, 4, 0.005, 0.01
    rows, cols, vals = _cells_by_column(nr, nc, 1.1, B, steps, 47)
    W, H = wl.uniform_table(nr, d, -0.1, 0.1, 7), wl.uniform_table(nc, d, -0.1, 0.1, 8)
    tw, th = dev(W), dev(H)
    ctx = nb.nups_init([tw, th], [d, d])
    hot_w, hot_h = np.arange(60, dtype=np.uint32), np.arange(30, dtype=np.uint32)
    nb.nups_set_hot_keys(ctx, 0, hot_w)
    nb.nups_set_hot_keys(ctx, 1, hot_h)
    nb.nups_set_update_clipping(ctx, 1.5)
    kr, kc, kv = dev_u32(rows), dev_u32(cols), dev(vals)
    rw, rh, sw, sh = W.copy(), H.copy(), np.zeros(2), np.zeros(2)
    for t in range(steps):
        nb.nups_step(ctx, nb.make_batch(nb.NUPS_TASK_MF, B, kr.data_ptr() + 4 * t * B, kc.data_ptr() + 4 * t * B,
                                        val=kv.data_ptr() + 4 * t * B, lr=lr, l2=l2))
        sl = slice(t * B, (t + 1) * B)
        orc.step_mf_clipped(rw, rh, d, rows[sl], cols[sl], vals[sl], lr, l2, hot_w, hot_h, 1.5, sw, sh)
    nb.nups_check(ctx)
    for table, ref in ((0, sw), (1, sh)):
        total, count = nb.nups_get_update_clipping(ctx, table)
        assert count == ref[1] and abs(total - ref[0]) <= 1e-5 * abs(ref[0])
    assert_table(tw.cpu().numpy(), rw, W, list(range(d)), 1e-4, "row factors", tol_update=1e-4)
    assert_table(th.cpu().numpy(), rh, H, list(range(d)), 1e-4, "column factors", tol_update=1e-4)
    nb.nups_destroy(ctx)


def test_steps_by_column_with_replicas():
    nr, nc, d, B, steps, R = 10_000, 1_000, 250, 4_096, 3, 4
    rows, cols, vals = _cells_by_column(nr, nc, 1.1, B, steps, 53)
    W, H = wl.uniform_table(nr, d, -0.1, 0.1, 9), wl.uniform_table(nc, d, -0.1, 0.1, 10)
    hot_w, hot_h = np.arange(100, dtype=np.uint32), np.arange(50, dtype=np.uint32)
    tw, th = dev(W), dev(H)
    ctx = nb.nups_init([tw, th], [d, d])
    nb.nups_set_hot_keys(ctx, 0, hot_w)
    nb.nups_set_hot_keys(ctx, 1, hot_h)
    nb.nups_set_replicas(ctx, R)
    kr, kc, kv = dev_u32(rows), dev_u32(cols), dev(vals)
    We, He = rep.extend_table(W, hot_w, R), rep.extend_table(H, hot_h, R)
    W0, H0 = We.copy(), He.copy()
    _run_steps(ctx, kr, kc, kv, B, steps, 4)
    for t in range(steps):
        sl = slice(t * B, (t + 1) * B)
        rep.step_mf_replicated(We, He, d, rows[sl], cols[sl], vals[sl], 0.005, 0.01, nr, nc, hot_w, hot_h, R)
    cols_ = list(range(d))
    assert_table(_extended(ctx, 0, tw), We, W0, cols_, 1e-4, "row factors and replicas", tol_update=1e-4)
    assert_table(_extended(ctx, 1, th), He, H0, cols_, 1e-4, "column factors and replicas", tol_update=1e-4)
    nb.nups_sync_replicas(ctx)
    rep.sync_replicas(We, nr, hot_w, R, d)
    rep.sync_replicas(He, nc, hot_h, R, d)
    assert_table(_extended(ctx, 1, th), He, H0, cols_, 1e-4, "column factors after synchronisation", tol_update=1e-4)
    nb.nups_destroy(ctx)
