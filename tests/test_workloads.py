"""The seeded input generators (no method arithmetic): shapes and the structure the recipes promise (CPU only)."""
import numpy as np

from paper_2104_00501_amd import workloads as wl


def test_window_pairs_count_and_order():
    toks = np.arange(20, dtype=np.uint32)
    c, o = wl.window_pairs(toks, 2, 0, wl.num_window_pairs(20, 2))
    assert len(c) == (20 - 4) * 4
    assert c[:4].tolist() == [2, 2, 2, 2] and o[:4].tolist() == [0, 1, 3, 4]


def test_zipf_stream_is_seeded_and_skewed():
    a, b = wl.zipf_stream(1000, 1.0, 50_000, 7), wl.zipf_stream(1000, 1.0, 50_000, 7)
    assert np.array_equal(a, b) and a.max() < 1000
    counts = np.bincount(a, minlength=1000)
    assert counts[0] > counts[9] > counts[99]              # key = rank - 1: key 0 is the most frequent
    assert abs(counts[0] / 50_000 - wl.zipf_pmf(1000, 1.0)[0]) < 0.01


def test_by_column_visiting_order():
    # Section 5.1: nodes by row, workers by column, each worker column by column in random order
    rows, cols, vals = wl.mf_cells(20_000, 3_000, 1.1, 120_000, 3)
    batch, nodes, per_node = 2048, 8, 8
    r, c, v = wl.mf_visit_by_column(rows, cols, vals, batch, 5, nodes, per_node)
    steps, per = len(r) // batch, batch // (nodes * per_node)
    assert steps >= 10 and len(r) == steps * batch
    cells = lambda a, b, x: sorted(zip(a.tolist(), b.tolist(), x.tolist()))
    pool = cells(rows, cols, vals)
    picked = cells(r, c, v)
    it = iter(pool)
    assert all(any(p == q for q in it) for p in picked)    # a sub-multiset of the input cells (both sorted)
    r3, c3 = r.reshape(steps, nodes * per_node, per), c.reshape(steps, nodes * per_node, per)
    for w in range(nodes * per_node):
        assert np.all(r3[:, w] % nodes == w // per_node) and np.all(c3[:, w] % per_node == w % per_node)
        seq = c3[:, w].ravel()                             # the worker's cells in the order it visits them
        runs = seq[np.concatenate([[True], seq[1:] != seq[:-1]])]
        assert len(np.unique(runs)) == len(runs)           # every column is visited in one go
    # locality: a batch touches far fewer distinct columns than the same cells in generation order
    assert len(np.unique(c[:batch])) < len(np.unique(cols[:batch])) / 2
    # seeded
    r2, c2, v2 = wl.mf_visit_by_column(rows, cols, vals, batch, 5, nodes, per_node)
    assert np.array_equal(r, r2) and np.array_equal(c, c2) and np.array_equal(v, v2)
