"""Oracle of the steps with stale replicas of the hot keys (Section 3.2: hot-spot keys are replicated on every
node, a node's workers read and update the node's replica, and the replicas are synchronised periodically by
exchanging the updates accumulated since the last synchronisation; Section 5.7 varies how often).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.  Plain numpy around the plain steps of nups_oracle.c.

Reading for one device (the paper's nodes become R parts of the minibatch):
 * the examples of a step are cut into R contiguous parts, example e of B belongs to part e * R // B;
 * every hot key has R replicas besides its row in the table (the base: the value at the last synchronisation);
   part r reads replica r wherever it accesses the key, and the part's summed gradient for the key updates
   replica r alone; keys that are not hot are shared by all parts, exactly as in the plain step;
 * the paper bounds staleness by time (a background thread synchronises every few milliseconds); here the caller
   synchronises after a number of steps of its choosing.  Synchronising adds every replica's accumulated update
   (replica - base) to the base, in replica order, and sets base and all replicas to the result.

A replica is nothing but one more row, so the state is an EXTENDED table of num_keys + R * H rows (H hot keys, hot
key number s of part r in row num_keys + r * H + s), a step is the plain step on remapped keys, and the only new
arithmetic is the synchronisation.
"""

from __future__ import annotations

import numpy as np

from . import oracle as orc


def hot_slots(num_keys: int, hot_keys) -> np.ndarray:
    """Position of each key in the hot list, -1 for keys that are not hot."""
    slot = np.full(num_keys, -1, dtype=np.int64)
    hot = np.asarray(hot_keys, dtype=np.int64)
    assert len(np.unique(hot)) == len(hot) and (len(hot) == 0 or (hot.min() >= 0 and hot.max() < num_keys))
    slot[hot] = np.arange(len(hot))
    return slot


def extend_table(table: np.ndarray, hot_keys, R: int) -> np.ndarray:
    """The table followed by R copies of its hot rows (every replica starts from the base)."""
    hot = np.asarray(hot_keys, dtype=np.int64)
    return np.ascontiguousarray(np.concatenate([table] + [table[hot]] * R, axis=0))


def part_of(example, B: int, R: int):
    """Part of the minibatch that an example belongs to: R contiguous parts."""
    return np.asarray(example, dtype=np.int64) * R // B


def remap_keys(keys, examples, B: int, num_keys: int, slot: np.ndarray, R: int) -> np.ndarray:
    """The row that each access really goes to: replica part_of(example) of a hot key, the key itself otherwise."""
    keys = np.asarray(keys, dtype=np.int64)
    H = int((slot >= 0).sum())
    s = slot[keys]
    return np.where(s >= 0, num_keys + part_of(examples, B, R) * H + s, keys).astype(np.uint32)


def step_sgns_replicated(In_ext, Out_ext, dim, center, context, negs, K, lr, V_in, V_out, hot_in, hot_out, R):
    """One word-vector step on extended tables (in place); center words index the input table's hot set, context
    words and negatives the output table's.  Returns the loss."""
    B = len(center)
    e = np.arange(B)
    c = remap_keys(center, e, B, V_in, hot_slots(V_in, hot_in), R)
    o = remap_keys(context, e, B, V_out, hot_slots(V_out, hot_out), R)
    ng = remap_keys(negs, np.repeat(e, K), B, V_out, hot_slots(V_out, hot_out), R)
    return orc.step_sgns(In_ext, Out_ext, dim, c, o, ng, K, lr)[0]


def step_mf_replicated(W_ext, H_ext, dim, rows, cols, vals, lr, l2, n_rows, n_cols, hot_rows, hot_cols, R):
    """One factorisation step on extended tables (in place).  Returns the loss."""
    B = len(rows)
    e = np.arange(B)
    r = remap_keys(rows, e, B, n_rows, hot_slots(n_rows, hot_rows), R)
    c = remap_keys(cols, e, B, n_cols, hot_slots(n_cols, hot_cols), R)
    return orc.step_mf(W_ext, H_ext, dim, r, c, vals, lr, l2)[0]


def sync_replicas(ext: np.ndarray, num_keys: int, hot_keys, R: int, dim: int) -> None:
    """base <- fl32(base + sum over replicas, in replica order, of (replica - base)), in fp64; every replica <- base."""
    hot = np.asarray(hot_keys, dtype=np.int64)
    H = len(hot)
    for s in range(H):
        base = ext[hot[s], :dim].astype(np.float64)
        total = base.copy()
        for r in range(R):
            total += ext[num_keys + r * H + s, :dim].astype(np.float64) - base
        new = total.astype(np.float32)
        ext[hot[s], :dim] = new
        for r in range(R):
            ext[num_keys + r * H + s, :dim] = new
