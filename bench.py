#!/usr/bin/env python3
"""Throughput of the sparse-SGD minibatch step on one MI355X.

Default workload: the large skip-gram configuration -- 1M keys, d = 300 (rows padded to 320
floats), 3 negatives per pair from unigram^0.75 under BOUNDED sample reuse (U = 4, pools of 250),
batches of 16,384 (center, context) pairs cut in stream order from an i.i.d. Zipf(1.0) token
stream with window 5, learning rate 0.025 linearly decayed.  One step = draw negatives, build the
per-key aggregation structure, score + gradient, aggregate and push, all inside the timed region;
inputs (example arrays, tables, alias table) are resident in HBM before timing starts.  Steps are
software-pipelined: the key-only halves of steps t+1 .. t+3 are enqueued before step t runs (--depth).

Other workloads (--workload): the small skip-gram configuration, matrix factorisation
(10M x 1M, rank 100, 65,536 cells per step) and ComplEx (4.6M entities, d = 500, 1,024 triples
with 50+50 uniform negatives per step, AdaGrad).

--clip F runs an SGD workload with the updates of its hot keys clipped at F times their mean norm
(Section 5.1 of the paper uses 2); the default is the plain summed-gradient step.

Prints one JSON line: positive examples/s, the roofline figure of the dominant kernel and the
CPU oracle timed on a bounded prefix of the same workload.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def progress(text):
    """One line on stderr per finished part of the run (the JSON line on stdout stays the only output there)."""
    print("bench: " + text, file=sys.stderr, flush=True)


def dev_keys(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint32).view(np.int32)).cuda()


class Sgns:
    """Skip-gram with negative sampling; tables 0/1 = input/output vectors."""

    def __init__(self, name, V, d, K, U, G, B, window, s, lr0, stream_tokens, seed, scheme=None, hot=None,
                 decay=True):
        self.name, self.V, self.d, self.K, self.U, self.G, self.B = name, V, d, K, U, G, B
        self.window, self.s, self.lr0, self.stream_tokens, self.seed = window, s, lr0, stream_tokens, seed
        self.scheme = scheme or ("BOUNDED" if U > 1 else "CONFORM")
        self.hot, self.decay = hot, decay       # hot: None = decided per step, else the top-`hot` keys are declared
        self.clip = 0.0                         # factor of the norm clipping of hot-key updates, 0 = off
        self.replicas, self.sync_every = 0, 1   # stale replicas of the hot keys (paper Section 3.2), 0 = off
        self.unit = "pairs"

    def setup(self, nb, wl, total_steps):
        import torch
        B, window = self.B, self.window
        n_tokens = min(self.stream_tokens, total_steps * B // (2 * window) + 2 * window + 2)
        toks = wl.zipf_stream(self.V, self.s, n_tokens, self.seed)
        self.centers, self.contexts = wl.window_pairs(toks, window, 0, total_steps * B)
        total_steps = len(self.centers) // B
        self.weights = wl.expected_unigram_weights(self.V, self.s, self.stream_tokens)
        self.stride = wl.padded_stride(self.d)
        if self.V * self.stride * 4 > (2 << 30):      # large tables are filled on the device
            g = torch.Generator(device="cuda").manual_seed(self.seed)
            tin = torch.zeros((self.V, self.stride), dtype=torch.float32, device="cuda")
            tin[:, :self.d] = (torch.rand((self.V, self.d), generator=g, device="cuda") - 0.5) / self.d
            self.tables = [tin, torch.zeros_like(tin)]
            self.In = self.Out = None                  # host copies are made when the oracle leg asks for them
        else:
            self.In, self.Out = wl.sgns_tables(self.V, self.d, self.seed)
            self.tables = [torch.from_numpy(self.In).cuda(), torch.from_numpy(self.Out).cuda()]
        self.kc, self.ko = dev_keys(self.centers), dev_keys(self.contexts)
        self.ctx = nb.nups_init(self.tables, [self.d, self.d])
        code = {"CONFORM": nb.NUPS_CONFORM, "BOUNDED": nb.NUPS_BOUNDED, "LONGTERM": nb.NUPS_LONGTERM,
                "NONCONFORM": nb.NUPS_NONCONFORM}[self.scheme]
        self.dist = nb.nups_register_distribution(self.ctx, 1, None if code == nb.NUPS_NONCONFORM else self.weights,
                                                  code, U=self.U, G=self.G, P=1_000_000, R=16, seed=self.seed)
        if self.hot is not None:                 # keys are frequency ranks: the top-k keys are 0..k-1
            for table in (0, 1):
                nb.nups_set_hot_keys(self.ctx, table, np.arange(self.hot, dtype=np.uint32))
        if self.clip > 0.0:
            nb.nups_set_update_clipping(self.ctx, self.clip)
        if self.replicas > 0:
            nb.nups_set_replicas(self.ctx, self.replicas)
        epoch_steps = max(1, wl.num_window_pairs(self.stream_tokens, window) // B)
        self.lrs = [float(wl.linear_lr(self.lr0, t, epoch_steps)) if self.decay else self.lr0
                    for t in range(total_steps)]
        self.nb = nb
        return total_steps

    def prepare(self, t):
        nb, B = self.nb, self.B
        if self.scheme == "NONCONFORM":          # negatives are context words of other pairs of the batch
            nb.nups_set_local_keys(self.dist, self.ko.data_ptr() + 4 * t * B, self.ko.data_ptr() + 4 * t * B, B,
                                   self.K, self.K, B)
        batch = nb.make_batch(nb.NUPS_TASK_SGNS, B, self.kc.data_ptr() + 4 * t * B, self.ko.data_ptr() + 4 * t * B,
                              n_neg=self.K, lr=self.lrs[t], dist=self.dist, sample_step=t)
        return nb.nups_prepare_step(self.ctx, batch)

    def accesses(self):
        return self.B, self.B * (self.K + 1)

    def algorithmic_bytes(self, nu0, nu1):
        row, B, K = 4 * self.d, self.B, self.K
        return {"grad": (nu0 + nu1) * row + 4 * B * (2 + K) + 4 * B * (K + 1),     # rows read once; keys; coefficients
                "apply0": nu0 * row * 2 + 4 * B,                                    # input rows read + written
                "apply1": nu1 * row * 2 + 8 * B * (K + 1),                          # output rows read + written
                "step": (nu0 + nu1) * row * 2 + 4 * B * (2 + K)}

    def logical_bytes(self):
        return self.B * (2 + self.K) * 4 * self.d * 3

    def oracle_step(self, orc, t):
        if not hasattr(self, "alias"):
            self.alias = orc.alias_build(self.weights)
            if self.In is None:
                self.In, self.Out = [x.cpu().numpy() for x in self.tables_initial]
        B, K = self.B, self.K
        c, o = self.centers[t * B:(t + 1) * B], self.contexts[t * B:(t + 1) * B]
        if self.scheme == "BOUNDED":
            ng = orc.sample_bounded(self.alias, self.V, self.seed, 0, t, B * K, self.U, self.G)
        elif self.scheme == "LONGTERM":
            ng = orc.sample_longterm(self.alias, self.V, self.seed, 0, 1_000_000, 16, t * B * K, B * K)
        elif self.scheme == "NONCONFORM":
            ng = orc.sample_nonconform(o, o, K, K, B, self.seed, 0, t, B * K)
        else:
            ng = orc.sample_conform(self.alias, self.V, self.seed, 0, t, B * K)
        if self.clip > 0.0:
            if not hasattr(self, "clip_stats"):
                self.clip_stats = np.zeros(2), np.zeros(2)
            hot = np.arange(self.hot, dtype=np.uint32)
            orc.step_sgns_clipped(self.In, self.Out, self.d, c, o, ng, K, self.lrs[t], hot, hot, self.clip,
                                  *self.clip_stats)
        elif self.replicas > 0:
            from oracle import replicas as rep
            hot = np.arange(self.hot, dtype=np.uint32)
            if not hasattr(self, "ext"):
                self.ext = [rep.extend_table(self.In, hot, self.replicas), rep.extend_table(self.Out, hot, self.replicas)]
            rep.step_sgns_replicated(self.ext[0], self.ext[1], self.d, c, o, ng, K, self.lrs[t], self.V, self.V, hot, hot,
                                     self.replicas)
            if (t + 1) % self.sync_every == 0:
                for e in self.ext:
                    rep.sync_replicas(e, self.V, hot, self.replicas, self.d)
        else:
            orc.step_sgns(self.In, self.Out, self.d, c, o, ng, K, self.lrs[t])

    def config(self):
        return {"workload": self.name, "task": "SGNS", "num_keys": self.V, "dim": self.d, "row_stride": self.stride,
                "negatives": self.K, "hot_keys": "per step" if self.hot is None else self.hot,
                "scheme": {"BOUNDED": "BOUNDED U=%d G=%d" % (self.U, self.G), "LONGTERM": "LONG-TERM P=1e6 R=16"}.get(
                    self.scheme, self.scheme),
                "batch": self.B, "window": self.window, "zipf_s": self.s, "lr0": self.lr0, "pairs": "stream order",
                "update_clipping": self.clip or "off",
                "replicas": "%d, synchronised every %d steps" % (self.replicas, self.sync_every) if self.replicas else "off"}


class Mf:
    """Matrix factorisation; tables 0/1 = row / column factors."""

    def __init__(self, name, n_rows, n_cols, d, B, s, lr, l2, seed, by_column=False):
        self.name, self.n_rows, self.n_cols, self.d, self.B, self.s = name, n_rows, n_cols, d, B, s
        self.lr, self.l2, self.seed = lr, l2, seed
        self.by_column = by_column              # cells in the paper's visiting order instead of generation order
        self.hot, self.clip = None, 0.0         # declared hot rows / columns (top-k by frequency rank); clipping factor
        self.unit = "cells"

    def setup(self, nb, wl, total_steps):
        import torch
        B = self.B
        if self.by_column:      # 64 workers, each column by column; the least loaded worker ends the run
            cells = wl.mf_cells(self.n_rows, self.n_cols, self.s, int(2.5 * total_steps * B), self.seed)
            progress("%d cells generated" % len(cells[0]))
            self.rows, self.cols, self.vals = wl.mf_visit_by_column(*cells, B, self.seed + 3)
            progress("cells put in the workers' by-column visiting order")
            assert len(self.rows) >= total_steps * B, "not enough cells for the requested steps"
        else:
            self.rows, self.cols, self.vals = wl.mf_cells(self.n_rows, self.n_cols, self.s, total_steps * B, self.seed)
        self.stride = wl.padded_stride(self.d)
        g = torch.Generator(device="cuda").manual_seed(self.seed)

        def table(n):
            t = torch.zeros((n, self.stride), dtype=torch.float32, device="cuda")
            t[:, :self.d] = torch.rand((n, self.d), generator=g, device="cuda") * 0.2 - 0.1
            return t

        self.tables = [table(self.n_rows), table(self.n_cols)]
        progress("factor tables initialised on the device")
        self.kr, self.kcol = dev_keys(self.rows), dev_keys(self.cols)
        self.kv = torch.from_numpy(self.vals).cuda()
        self.ctx = nb.nups_init(self.tables, [self.d, self.d])
        if self.hot is not None:                 # keys are frequency ranks: the top-k keys are 0..k-1
            for table in (0, 1):
                nb.nups_set_hot_keys(self.ctx, table, np.arange(self.hot, dtype=np.uint32))
        if self.clip > 0.0:
            nb.nups_set_update_clipping(self.ctx, self.clip)
        self.nb = nb
        return total_steps

    def prepare(self, t):
        nb, B = self.nb, self.B
        batch = nb.make_batch(nb.NUPS_TASK_MF, B, self.kr.data_ptr() + 4 * t * B, self.kcol.data_ptr() + 4 * t * B,
                              val=self.kv.data_ptr() + 4 * t * B, lr=self.lr, l2=self.l2)
        return nb.nups_prepare_step(self.ctx, batch)

    def accesses(self):
        return self.B, self.B

    def note_structure(self, t, table, keys, counts):
        """Rows / columns that the gradient kernel updates itself: rows with one access in step t, columns whose
        cells of step t all stand in one run (consecutive cells inside one block of 16 cells)."""
        if self.clip > 0.0:         # with clipping on every update goes through the update kernel
            return
        self.alone = getattr(self, "alone", [[], []])
        if table == 0 or self.stride < 256:      # narrow rows: columns are treated like rows (kMfRunsFromNV4)
            self.alone[table].append(int((counts == 1).sum()))
            return
        c = self.cols[t * self.B:(t + 1) * self.B]
        head = np.ones(len(c), dtype=bool)
        head[1:] = c[1:] != c[:-1]
        head[::16] = True
        run_len = np.diff(np.append(np.flatnonzero(head), len(c)))
        whole = run_len == counts[np.searchsorted(keys, c[head])]
        self.alone[1].append(int(whole.sum()))

    def algorithmic_bytes(self, nu0, nu1):
        row, B = 4 * self.d, self.B
        a0, a1 = [float(np.mean(x)) if x else 0.0 for x in getattr(self, "alone", [[], []])]
        # every distinct row read once and written once: written by the gradient kernel if it updates the row itself
        # (note_structure), by the update kernel (which reads it again) otherwise
        return {"grad": (nu0 + nu1) * row + (a0 + a1) * row + 12 * B,
                "apply0": (nu0 - a0) * row * 2 + 4 * B, "apply1": (nu1 - a1) * row * 2 + 4 * B,
                "step": (nu0 + nu1) * row * 2 + 12 * B}

    def logical_bytes(self):
        return self.B * 2 * 4 * self.d * 3

    def oracle_step(self, orc, t):
        if not hasattr(self, "host"):
            self.host = [x.cpu().numpy() for x in self.tables_initial]
        B = self.B
        sl = slice(t * B, (t + 1) * B)
        if self.clip > 0.0:
            if not hasattr(self, "clip_stats"):
                self.clip_stats = np.zeros(2), np.zeros(2)
            hot = np.arange(self.hot, dtype=np.uint32)
            orc.step_mf_clipped(self.host[0], self.host[1], self.d, self.rows[sl], self.cols[sl], self.vals[sl],
                                self.lr, self.l2, hot, hot, self.clip, *self.clip_stats)
        else:
            orc.step_mf(self.host[0], self.host[1], self.d, self.rows[sl], self.cols[sl], self.vals[sl], self.lr,
                        self.l2)

    def config(self):
        return {"workload": self.name, "task": "MF", "rows": self.n_rows, "cols": self.n_cols, "dim": self.d,
                "row_stride": self.stride, "batch": self.B, "zipf_s": self.s, "lr": self.lr, "l2": self.l2,
                "hot_keys": "per step" if self.hot is None else self.hot, "update_clipping": self.clip or "off",
                "cells": "64 workers, each column by column" if self.by_column else "generation order"}


class Kge:
    """ComplEx with AdaGrad; tables 0/1 = entities / relations, each with a state table."""

    def __init__(self, name, n_ent, n_rel, d, B, nh, nt, lr, eps, seed):
        self.name, self.n_ent, self.n_rel, self.d, self.B, self.nh, self.nt = name, n_ent, n_rel, d, B, nh, nt
        self.lr, self.eps, self.seed = lr, eps, seed
        self.unit = "triples"

    def setup(self, nb, wl, total_steps):
        import torch
        B = self.B
        self.s, self.r, self.o = wl.kge_triples(self.n_ent, self.n_rel, total_steps * B, self.seed)
        self.stride = wl.padded_stride(self.d)
        if self.stride % 128:
            self.stride += 64
        g = torch.Generator(device="cuda").manual_seed(self.seed)
        half = self.d // 2

        def table(n):
            t = torch.zeros((n, self.stride), dtype=torch.float32, device="cuda")
            t[:, :half] = torch.rand((n, half), generator=g, device="cuda") * 0.2 - 0.1
            t[:, self.stride // 2:self.stride // 2 + half] = torch.rand((n, half), generator=g, device="cuda") * 0.2 - 0.1
            return t

        self.tables = [table(self.n_ent), table(self.n_rel)]
        self.states = [torch.zeros_like(self.tables[0]), torch.zeros_like(self.tables[1])]
        for st in self.states:                                  # a warmed-up accumulator on the logical lanes
            st[:, :half] = 1e-3
            st[:, self.stride // 2:self.stride // 2 + half] = 1e-3
        self.ks, self.kr, self.ko = dev_keys(self.s), dev_keys(self.r), dev_keys(self.o)
        self.ctx = nb.nups_init(self.tables, [self.d, self.d])
        nb.nups_set_state(self.ctx, 0, self.states[0])
        nb.nups_set_state(self.ctx, 1, self.states[1])
        self.dist = nb.nups_register_distribution(self.ctx, 0, None, nb.NUPS_CONFORM, seed=self.seed)
        self.nb = nb
        return total_steps

    def prepare(self, t):
        nb, B = self.nb, self.B
        batch = nb.make_batch(nb.NUPS_TASK_KGE, B, self.ks.data_ptr() + 4 * t * B, self.kr.data_ptr() + 4 * t * B,
                              k2=self.ko.data_ptr() + 4 * t * B, n_neg=self.nh, n_neg2=self.nt, lr=self.lr,
                              eps=self.eps, dist=self.dist, sample_step=t)
        return nb.nups_prepare_step(self.ctx, batch)

    def accesses(self):
        return self.B * (2 + self.nh + self.nt), self.B

    def note_structure(self, t, table, keys, counts):
        """Entities that the gradient kernel updates itself: accessed once in step t, by a negative."""
        if table != 0:
            return
        sl = slice(t * self.B, (t + 1) * self.B)
        once = keys[counts == 1]
        self.alone = getattr(self, "alone", []) + [int(np.isin(once, np.concatenate([self.s[sl], self.o[sl]]),
                                                               invert=True).sum())]

    def algorithmic_bytes(self, nu0, nu1):
        row, B, nn = 4 * self.d, self.B, self.nh + self.nt
        alone = float(np.mean(self.alone)) if getattr(self, "alone", None) else 0.0
        # value and state rows, read + written: by the gradient kernel for negatives that are their entity's only
        # access, by the update kernel for every other distinct row
        return {"grad": alone * row * 4 + (nu0 - alone + nu1) * row + 4 * B * (3 + nn) + 4 * B * nn,
                "apply0": (nu0 - alone) * row * 4 + 8 * B * nn,
                "apply1": nu1 * row * 4 + 4 * B,
                "step": (nu0 + nu1) * row * 4 + 4 * B * (3 + nn)}

    def logical_bytes(self):
        return self.B * (3 + self.nh + self.nt) * 4 * self.d * 5

    def oracle_step(self, orc, t):
        if not hasattr(self, "host"):
            self.host = [x.cpu().numpy() for x in self.tables_initial] + [x.cpu().numpy() for x in self.states_initial]
        B, nn = self.B, self.nh + self.nt
        sl = slice(t * B, (t + 1) * B)
        negs = orc.sample_conform(None, self.n_ent, self.seed, 0, t, B * nn)
        orc.step_kge(self.host[0], self.host[2], self.host[1], self.host[3], self.d, self.s[sl], self.r[sl],
                     self.o[sl], negs, self.nh, self.nt, self.lr, self.eps)

    def config(self):
        return {"workload": self.name, "task": "KGE (ComplEx, AdaGrad)", "entities": self.n_ent,
                "relations": self.n_rel, "dim": self.d, "row_stride": self.stride, "batch": self.B,
                "negatives": "%d subject + %d object, uniform" % (self.nh, self.nt), "lr": self.lr}


def _sweep_workloads():
    """The skew / technique / scheme grid: 500k keys, d = 200, 5 negatives, batches of 8,192 pairs."""
    out = {}
    for s_exp in (0.6, 1.0, 1.4):
        for hot in (0, 1000, 16000):
            for scheme, U in (("CONFORM", 1), ("BOUNDED", 16), ("LONGTERM", 1), ("NONCONFORM", 1)):
                name = "sweep_s%.1f_top%d_%s" % (s_exp, hot, scheme.lower())
                out[name] = (lambda n=name, s_=s_exp, h=hot, sc=scheme, u=U:
                             Sgns(n, 500_000, 200, 5, u, 250, 8192, 5, s_, 0.025, 200_000_000, 1005, scheme=sc, hot=h,
                                  decay=False))
    return out


WORKLOADS = {
    "sgns_1m_d300_bounded_u4": lambda: Sgns("sgns_1m_d300_bounded_u4", 1_000_000, 300, 3, 4, 250, 16_384, 5, 1.0,
                                            0.025, 1_000_000_000, 1004),
    "sgns_10k_d100_conform": lambda: Sgns("sgns_10k_d100_conform", 10_000, 100, 5, 1, 1, 4096, 2, 1.0, 0.025,
                                          1_000_000, 1001),
    "mf_10m_1m_d100": lambda: Mf("mf_10m_1m_d100", 10_000_000, 1_000_000, 100, 65_536, 0.8, 0.005, 0.01, 1002),
    "kge_4p6m_d500": lambda: Kge("kge_4p6m_d500", 4_600_000, 822, 500, 1024, 50, 50, 0.1, 1e-10, 1003),
}
# The paper's own shapes (Table 1, Section 5.1) where they differ from the configurations above: word vectors of
# dimension 1000 over 1.9M words under the untuned configuration's BOUNDED reuse (U = 16); factorisation of rank
# 1000 with Zipf(1.1) ids, visited by column; ComplEx with 100 + 100 negatives over 4.8M entities and 828 relations.
WORKLOADS.update({
    "sgns_1p9m_d1000_bounded_u16": lambda: Sgns("sgns_1p9m_d1000_bounded_u16", 1_900_000, 1000, 3, 16, 250, 16_384,
                                                5, 1.0, 0.025, 375_000_000, 1006),
    "mf_10m_1m_rank1000_by_column": lambda: Mf("mf_10m_1m_rank1000_by_column", 10_000_000, 1_000_000, 1000, 65_536,
                                               1.1, 0.005, 0.01, 1007, by_column=True),
    "mf_10m_1m_d100_by_column": lambda: Mf("mf_10m_1m_d100_by_column", 10_000_000, 1_000_000, 100, 65_536, 0.8,
                                           0.005, 0.01, 1002, by_column=True),
    "kge_4p8m_d500_neg100_100": lambda: Kge("kge_4p8m_d500_neg100_100", 4_818_679, 828, 500, 1024, 100, 100, 0.1,
                                            1e-10, 1008),
})
WORKLOADS.update(_sweep_workloads())


def kernel_sources_digest():
    """sha256 over the library's kernel sources, in name order."""
    import hashlib
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2104_00501_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the hardware-counter runs summarised in profiles/hbm_traffic.txt
    (fetch bytes already scaled by the calibration copy), or None when no line matches the workload, the
    kernel and the present kernel sources: counters taken before a kernel changed say nothing about it."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    digest = kernel_sources_digest()
    with open(path) as f:
        for line in f:
            parts = line.split()
            if len(parts) == 5 and not line.startswith("#") and parts[0] == workload and parts[1] == kernel \
                    and parts[4] == digest:
                return float(parts[2]) + float(parts[3])
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="sgns_1m_d300_bounded_u4", choices=sorted(WORKLOADS))
    ap.add_argument("--depth", type=int, default=None,
                    help="steps prepared ahead of the one that runs (default 3; 4 for matrix factorisation and "
                         "with --deterministic)")
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps to time (-1: about 15 s worth, 0: skip)")
    ap.add_argument("--clip", type=float, default=0.0,
                    help="SGD workloads: clip hot-key updates at this factor times their mean norm (0: off); "
                         "declares the 1,000 most frequent keys of each table as hot if the workload declares none")
    ap.add_argument("--replicas", type=int, default=0,
                    help="skip-gram workloads: this many stale replicas of each hot key (paper Section 3.2), one per "
                         "contiguous part of the batch; declares the 1,000 most frequent keys hot if none are declared")
    ap.add_argument("--deterministic", action="store_true",
                    help="sum every key's contributions in a fixed order (results bit-identical from run to run)")
    ap.add_argument("--sync-every", type=int, default=8, help="steps between two synchronisations of the replicas")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2
    from paper_2104_00501_amd.build import ensure_built
    ensure_built()          # loads the in-tree library; compiles it only if it is not there

    import torch

    from paper_2104_00501_amd import binding as nb
    from paper_2104_00501_amd import workloads as wl

    torch.cuda.set_device(0)
    w = WORKLOADS[args.workload]()
    if args.depth is None:
        args.depth = 4 if isinstance(w, Mf) or args.deterministic else 3   # deterministic mode: two more phases per step
    if args.clip > 0.0:
        if isinstance(w, Kge):
            print("--clip applies to the SGD workloads; the AdaGrad steps are never clipped", file=sys.stderr)
            return 2
        w.clip = args.clip
        if not w.hot:
            w.hot = 1000
    n_windows = 5                                    # further timed windows after the headline region
    window = max(20, min(args.steps, 100))
    if args.replicas > 0:
        if not isinstance(w, Sgns) or args.clip > 0.0:
            print("--replicas applies to the skip-gram workloads, without --clip", file=sys.stderr)
            return 2
        w.replicas, w.sync_every = args.replicas, max(1, args.sync_every)
        if not w.hot:
            w.hot = 1000
    total_steps = w.setup(nb, wl, args.warmup + args.steps + n_windows * window)
    steps = args.steps
    assert total_steps >= args.warmup + steps, "not enough examples for the requested steps"
    progress("workload %s set up (%d steps of input resident)" % (args.workload, total_steps))
    n_windows = min(n_windows, (total_steps - args.warmup - steps) // window)
    ctx, B = w.ctx, w.B
    if args.deterministic:
        nb.nups_set_deterministic(ctx, 1)
    if args.cpu_steps != 0 and getattr(w, "In", None) is None:   # the oracle starts from the same initial tables
        w.tables_initial = [t.clone() for t in w.tables]
        if hasattr(w, "states"):
            w.states_initial = [t.clone() for t in w.states]

    class Pipeline:
        """Software pipeline: steps t+1 .. t+depth are prepared before step t runs, so that sampling and the
        aggregation structure of later steps ride in the launches of step t and its neighbours."""

        def __init__(self, first, last):
            self.next_run, self.next_prepare, self.last = first, first, last
            self.queue = []
            self.fill()

        def fill(self):
            while self.next_prepare < min(self.next_run + args.depth + 1, self.last):
                self.queue.append(w.prepare(self.next_prepare))
                self.next_prepare += 1

        def run(self, count):
            for _ in range(count):
                nb.nups_step_prepared(ctx, self.queue.pop(0))
                self.next_run += 1
                if getattr(w, "replicas", 0) and self.next_run % w.sync_every == 0:
                    nb.nups_sync_replicas(ctx)              # inside the timed region: part of the method's cost
                self.fill()

    def run(first, count):                           # a pipeline of its own (the per-kernel pass)
        Pipeline(first, first + count).run(count)

    # ---- warm-up, then the timed region: one pipeline runs through both, so that the timed steps find their
    # preparatory work carried by the launches before them, as in steady state --------------------------------
    pipe = Pipeline(0, args.warmup + steps + n_windows * window)
    pipe.run(args.warmup)
    nb.nups_check(ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipe.run(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    nb.nups_check(ctx)
    ms_per_step = 1e3 * elapsed / steps
    value = steps * B / elapsed
    window_ms = []
    for _ in range(n_windows):                       # the same measurement again, several times: its spread
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        pipe.run(window)
        torch.cuda.synchronize()
        window_ms.append(1e3 * (time.perf_counter() - t1) / window)
    nb.nups_check(ctx)
    finite = all(bool(torch.isfinite(t).all().item()) for t in w.tables)
    total_steps = args.warmup + steps + n_windows * window
    progress("timed region done: %.4f ms per step over %d steps, %d further windows" % (ms_per_step, steps, n_windows))

    # ---- per-kernel pass: the last steps again, unpipelined, HIP events around every phase on its stream ---
    n_prof = min(steps, 64)
    first_prof = total_steps - n_prof
    nb.nups_profile(ctx, True)
    n0, n1 = w.accesses()
    uk = torch.zeros(max(n0, n1), dtype=torch.int32, device="cuda")
    uc = torch.zeros(max(n0, n1), dtype=torch.int32, device="cuda")
    nu0 = nu1 = 0
    for t in range(first_prof, first_prof + n_prof):
        run(t, 1)
        for table in (0, 1):                                # distinct rows per step, for the algorithmic bytes
            n_t = nb.nups_debug_structure(ctx, table, uk, uc)
            if hasattr(w, "note_structure"):
                w.note_structure(t, table, uk[:n_t].cpu().numpy().view(np.uint32),
                                 uc[:n_t].cpu().numpy().view(np.uint32))
            nu0, nu1 = (nu0 + n_t, nu1) if table == 0 else (nu0, nu1 + n_t)
    nu0 /= n_prof
    nu1 /= n_prof
    phases = {}
    for p in range(nb.NUPS_PHASE_COUNT):
        ms, n = nb.nups_profile_read(ctx, p)
        if n:
            phases[nb.nups_phase_name(p)] = ms / n_prof
    nb.nups_profile(ctx, False)
    # what a pair of HIP events reads with nothing between them, on the stream the kernels run on: a bracket around
    # one launch includes this much besides the kernel (rocprofv3's per-dispatch durations do not)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    empty_ms = []
    for _ in range(51):
        ev0.record()
        ev1.record()
        torch.cuda.synchronize()
        empty_ms.append(ev0.elapsed_time(ev1))
    empty_bracket_ms = float(np.median(empty_ms))
    progress("per-kernel pass done (%d unpipelined steps)" % n_prof)

    # a plain copy of known size through the library's own gather kernel (rows 0..n-1 in order): the
    # reference that hardware byte counters are scaled with
    n_cal = min(int(w.tables[0].shape[0]), 262_144)
    cal_keys = torch.arange(n_cal, dtype=torch.int32, device="cuda")
    cal_out = torch.empty((n_cal, w.stride), dtype=torch.float32, device="cuda")
    nb.nups_pull(ctx, 0, cal_keys, n_cal, cal_out)
    torch.cuda.synchronize()
    # the same number of rows at uniformly random keys (the second launch of the gather kernel, for the same
    # scaling on a random gather), then both again several times for the gather's own rate
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    rnd_keys = torch.randint(0, int(w.tables[0].shape[0]), (n_cal,), dtype=torch.int32, device="cuda", generator=gen)
    nb.nups_pull(ctx, 0, rnd_keys, n_cal, cal_out)
    torch.cuda.synchronize()
    pull = {"rows": n_cal, "bytes_per_call": 2 * n_cal * w.stride * 4}
    for name, keys in (("in_order", cal_keys), ("random", rnd_keys)):
        t1 = time.perf_counter()
        for _ in range(10):
            nb.nups_pull(ctx, 0, keys, n_cal, cal_out)
        torch.cuda.synchronize()
        pull[name + "_GBps"] = 10 * pull["bytes_per_call"] / (time.perf_counter() - t1) / 1e9
    del cal_out

    # Algorithmic bytes under snapshot semantics: every distinct touched row is read once and written
    # once (4 * d bytes each way; twice that with optimiser state), plus the key arrays.
    alg = w.algorithmic_bytes(nu0, nu1)
    if "apply1" not in phases:        # both tables are updated by one launch, timed as "apply0"
        alg["apply0"] += alg.pop("apply1")
    dominant = max((p for p in ("grad", "apply0", "apply1") if p in phases and p in alg), key=lambda p: phases[p])
    dom_ms = phases[dominant]
    achieved = alg[dominant] / (dom_ms * 1e-3) / 1e9
    step_traffic = recorded_traffic(args.workload, "step")     # all kernels of a step, by the same counters
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": recorded_traffic(args.workload, dominant),
                "algorithmic_bytes_per_launch": alg[dominant], "kernel_ms": dom_ms,
                "empty_event_bracket_ms": empty_bracket_ms,
                "per_kernel_GBps": {p: alg[p] / (phases[p] * 1e-3) / 1e9 for p in ("grad", "apply0", "apply1")
                                    if p in phases and p in alg},
                "whole_step_algorithmic_GBps": alg["step"] / (ms_per_step * 1e-3) / 1e9,
                "whole_step_traffic": step_traffic,
                "whole_step_traffic_GBps": None if step_traffic is None else step_traffic / (ms_per_step * 1e-3) / 1e9,
                "whole_step_logical_GBps": w.logical_bytes() / (ms_per_step * 1e-3) / 1e9,
                "distinct_rows_per_step": {"table0": nu0, "table1": nu1}}

    # ---- CPU baseline: the oracle, as it stands, on a prefix of the same steps -------------------
    cpu = None
    if args.cpu_steps != 0:
        from oracle import oracle as orc
        n_cpu = args.cpu_steps if args.cpu_steps > 0 else 10 ** 9
        progress("oracle: copying the initial tables to the host")
        w.oracle_step(orc, 0)                                # first call also builds tables / alias table
        progress("oracle: first step done, timing further steps")
        done, t_cpu = 1, time.perf_counter()
        t_said = t_cpu
        while done < min(n_cpu + 1, total_steps):
            w.oracle_step(orc, done)
            done += 1
            if time.perf_counter() - t_said > 30.0:
                t_said = time.perf_counter()
                progress("oracle: %d steps timed" % (done - 1))
            if args.cpu_steps < 0 and time.perf_counter() - t_cpu > 15.0:
                break
        dt = time.perf_counter() - t_cpu
        cpu = {"value": (done - 1) * B / dt, "unit": "positive examples/s", "cores": 1, "kind": "oracle",
               "sample": "steps 1..%d of the same workload (%d %s), single thread, %.1f s"
                         % (done - 1, (done - 1) * B, w.unit, dt),
               "host_cores_available": os.cpu_count()}

    out = {
        "metric": "positive examples/sec per step (pull+grad+push)", "value": value, "unit": "positive examples/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": w.config(), "roofline": roofline, "phases_ms_per_step": phases, "cpu_baseline": cpu,
        "finite": finite, "gather_kernel": pull, "deterministic": bool(args.deterministic),
        "windows_ms_per_step": {"steps_per_window": window, "median": float(np.median(window_ms)) if window_ms else None,
                                "min": min(window_ms) if window_ms else None, "max": max(window_ms) if window_ms else None},
    }
    if not finite:
        out["finite_note"] = ("tables overflow at this configuration's learning rate with summed minibatch gradients; "
                              "the oracle overflows in the same way; kernel timing does not depend on the values (--clip 2 "
                              "runs the same workload with the paper's remedy, norm clipping of hot-key updates)")
    nb.nups_destroy(ctx)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
