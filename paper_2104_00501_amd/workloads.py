"""Seeded synthetic inputs shaped like the paper's three tasks (Section 5.1, Table 1).

This module only *generates data*: Zipf-skewed key streams, (center, context)
pair enumeration, observed matrix cells, triples, sampling weights and initial
table values.  It contains none of the method's arithmetic (no sampling scheme,
no loss, no update rule) and is the only module that both the CPU oracle's
tests and the GPU path's tests import, so that both sides see identical inputs.

Key ids are Zipf ranks minus one: key 0 is the most frequent key.
"""

from __future__ import annotations

import numpy as np

ROW_LANES = 64  # tables are stored with the row length padded to a multiple of 64 floats


def padded_stride(dim: int) -> int:
    """Row stride (in floats) of a table whose logical row length is ``dim``."""
    return ((int(dim) + ROW_LANES - 1) // ROW_LANES) * ROW_LANES


def zipf_pmf(num_keys: int, s: float) -> np.ndarray:
    """p_k proportional to (k+1)^-s over keys 0..num_keys-1, in fp64."""
    w = np.arange(1, num_keys + 1, dtype=np.float64) ** (-float(s))
    return w / w.sum()


def zipf_stream(num_keys: int, s: float, n: int, seed: int) -> np.ndarray:
    """n i.i.d. keys from Zipf(s) over num_keys keys (inverse-CDF draws), uint32."""
    rng = np.random.default_rng(seed)
    cdf = np.cumsum(zipf_pmf(num_keys, s))
    cdf[-1] = 1.0
    u = rng.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="right"), num_keys - 1).astype(np.uint32)


def num_window_pairs(num_tokens: int, window: int) -> int:
    """Number of (center, context) pairs of a token stream with a fixed window.

    Only centers with a full window on both sides are used, so the count is
    (num_tokens - 2*window) * 2*window.
    """
    return max(0, num_tokens - 2 * window) * 2 * window


def window_pairs(tokens: np.ndarray, window: int, first_pair: int, count: int):
    """Pairs first_pair .. first_pair+count-1 of the stream, in stream order.

    Pair p has its center at position window + p // (2*window); its context
    offset is the (p mod 2*window)-th entry of (-window..-1, +1..+window).
    Returns (center_keys, context_keys) as uint32 arrays.
    """
    w2 = 2 * window
    total = num_window_pairs(len(tokens), window)
    count = max(0, min(count, total - first_pair))
    p = np.arange(first_pair, first_pair + count, dtype=np.int64)
    t = window + p // w2
    j = p % w2
    off = np.where(j < window, j - window, j - window + 1)
    return tokens[t].astype(np.uint32), tokens[t + off].astype(np.uint32)


def unigram_weights(tokens: np.ndarray, num_keys: int, power: float = 0.75) -> np.ndarray:
    """Sampling weights count_k ** power (fp64); keys that never occur get weight 0."""
    counts = np.bincount(tokens, minlength=num_keys).astype(np.float64)
    return counts ** float(power)


def expected_unigram_weights(num_keys: int, s: float, num_tokens: float, power: float = 0.75) -> np.ndarray:
    """Weights (num_tokens * p_k) ** power for streams too long to materialise."""
    return (zipf_pmf(num_keys, s) * float(num_tokens)) ** float(power)


def uniform_table(num_keys: int, dim: int, lo: float, hi: float, seed: int) -> np.ndarray:
    """[num_keys, padded_stride(dim)] fp32 table, U(lo, hi) in the first dim lanes, 0 in the padding."""
    rng = np.random.default_rng(seed)
    t = np.zeros((num_keys, padded_stride(dim)), dtype=np.float32)
    t[:, :dim] = (rng.random((num_keys, dim), dtype=np.float32) * np.float32(hi - lo) + np.float32(lo))
    return t


def complex_table(num_keys: int, dim: int, lo: float, hi: float, seed: int) -> np.ndarray:
    """Table of complex rows: dim/2 real parts from float 0, dim/2 imaginary parts from float stride/2."""
    rng = np.random.default_rng(seed)
    stride = padded_stride(dim)
    if stride % 128:
        stride += ROW_LANES          # both halves have to be multiples of 64 floats
    half = dim // 2
    t = np.zeros((num_keys, stride), dtype=np.float32)
    t[:, :half] = rng.random((num_keys, half), dtype=np.float32) * np.float32(hi - lo) + np.float32(lo)
    t[:, stride // 2:stride // 2 + half] = (rng.random((num_keys, half), dtype=np.float32)
                                            * np.float32(hi - lo) + np.float32(lo))
    return t


def zero_table(num_keys: int, dim: int) -> np.ndarray:
    return np.zeros((num_keys, padded_stride(dim)), dtype=np.float32)


def sgns_tables(num_keys: int, dim: int, seed: int):
    """Input table U(-0.5/dim, 0.5/dim), output table zeros."""
    return uniform_table(num_keys, dim, -0.5 / dim, 0.5 / dim, seed), zero_table(num_keys, dim)


def _hashed_normals(ids: np.ndarray, salt: int, seed: int, width: int) -> np.ndarray:
    """[len(ids), width] standard normals that depend only on (seed, salt, id, column)."""
    with np.errstate(over="ignore"):
        def mix(z):
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            return z ^ (z >> np.uint64(31))
        base = (ids.astype(np.uint64)[:, None] * np.uint64(2 * width)
                + np.arange(2 * width, dtype=np.uint64)[None, :])
        h = mix(mix(base + np.uint64(0x9E3779B97F4A7C15) * np.uint64(seed * 1000003 + salt + 1)))
    u = ((h >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    return np.sqrt(-2.0 * np.log(u[:, :width])) * np.cos(2.0 * np.pi * u[:, width:])


def mf_cells(num_rows: int, num_cols: int, s: float, n: int, seed: int,
             hidden_rank: int = 10, noise: float = 0.1):
    """n observed cells: row and column ids i.i.d. Zipf(s) (duplicates kept), value =
    <a_row, b_col> + N(0, noise), with hidden factors a, b of hidden_rank entries each
    N(0, variance 1/sqrt(hidden_rank)) so that <a, b> has unit variance.

    The hidden factor of an id depends only on (seed, id), so any window of a
    long cell stream can be generated on its own.
    """
    rows = zipf_stream(num_rows, s, n, seed)
    cols = zipf_stream(num_cols, s, n, seed + 1)
    rng = np.random.default_rng(seed + 2)
    scale = float(hidden_rank) ** -0.25
    vals = np.empty(n, dtype=np.float64)
    for lo in range(0, n, 1 << 20):
        hi = min(n, lo + (1 << 20))
        a = _hashed_normals(rows[lo:hi], 11, seed, hidden_rank) * scale
        b = _hashed_normals(cols[lo:hi], 12, seed, hidden_rank) * scale
        vals[lo:hi] = np.einsum("nk,nk->n", a, b)
    vals = vals + noise * rng.standard_normal(n)
    return rows, cols, vals.astype(np.float32)


def mf_visit_by_column(rows: np.ndarray, cols: np.ndarray, vals: np.ndarray, batch: int, seed: int,
                       nodes: int = 8, workers_per_node: int = 8):
    """Reorders cells into the visiting order of the factorisation task (Section 5.1): cells are
    partitioned to nodes by row and to the workers of a node by column (here: id modulo the number
    of parts, so that the frequent ids, which are the small ones, spread evenly); each worker
    walks its cells column by column, columns in random order, the cells of a column in random
    order.  Batch t is the t-th slice of batch / (nodes * workers_per_node) cells of every
    worker, concatenated in worker order; the run ends when the first worker runs out of cells.
    Returns (rows, cols, vals) of steps * batch cells.
    """
    workers = nodes * workers_per_node
    assert batch % workers == 0, "the batch is shared evenly among the workers"
    per = batch // workers
    rng = np.random.default_rng(seed)
    n = len(rows)
    worker = (rows % nodes).astype(np.int64) * workers_per_node + (cols % workers_per_node).astype(np.int64)
    column_order = rng.permutation(int(cols.max()) + 1 if n else 1)
    order = np.lexsort((rng.random(n), column_order[cols], worker))   # by worker, column order, then at random
    counts = np.bincount(worker, minlength=workers)
    steps = int(counts.min()) // per
    starts = np.concatenate([[0], np.cumsum(counts)[:-1]])
    idx = (starts[None, :, None] + np.arange(steps, dtype=np.int64)[:, None, None] * per
           + np.arange(per, dtype=np.int64)[None, None, :])
    sel = order[idx.reshape(-1)]
    return rows[sel], cols[sel], vals[sel]


def kge_triples(num_entities: int, num_relations: int, n: int, seed: int,
                s_entity: float = 1.1, s_relation: float = 1.5):
    """n triples: head and tail i.i.d. Zipf(s_entity), relation i.i.d. Zipf(s_relation)."""
    heads = zipf_stream(num_entities, s_entity, n, seed)
    rels = zipf_stream(num_relations, s_relation, n, seed + 1)
    tails = zipf_stream(num_entities, s_entity, n, seed + 2)
    return heads, rels, tails


def top_keys_by_frequency(access_counts: np.ndarray, k: int) -> np.ndarray:
    """The k keys with the largest access count, ties broken by ascending key, uint32."""
    k = int(min(k, len(access_counts)))
    if k <= 0:
        return np.zeros(0, dtype=np.uint32)
    order = np.lexsort((np.arange(len(access_counts)), -np.asarray(access_counts, dtype=np.float64)))
    return order[:k].astype(np.uint32)


def linear_lr(lr0: float, step: int, total_steps: int) -> np.float32:
    """Linearly decayed learning rate lr0 * max(1e-4, 1 - step/total_steps), rounded to fp32."""
    return np.float32(float(lr0) * max(1e-4, 1.0 - float(step) / float(total_steps)))
