"""ctypes front end of the CPU oracle in nups_oracle.c.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
it is used by the tests, by the smoke check and by the CPU-baseline leg of the
benchmark.  It marshals numpy arrays into the C functions and adds nothing to
their arithmetic.
"""

from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nups_oracle.c")
_LIB = os.path.join(_HERE, "libnups_oracle.so")

CONFORM, BOUNDED, LONGTERM, NONCONFORM = 1, 2, 3, 4


def build(force: bool = False) -> str:
    """Compile nups_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.nor_distinct_keys.restype = C.c_int64
        _lib.nor_permute.restype = C.c_uint64
        for f in ("nor_loss_sgns", "nor_loss_mf", "nor_loss_kge", "nor_complex_score"):
            getattr(_lib, f).restype = C.c_double
    return _lib


def _p(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _u32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.uint32)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s failed with status %d" % (what, rc))


def _table(t):
    assert t.dtype == np.float32 and t.ndim == 2 and t.flags.c_contiguous
    return t


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().nor_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def words(seed, stream, dist_id, step, draw):
    out = np.zeros(4, dtype=np.uint32)
    lib().nor_words(C.c_uint64(seed), C.c_uint32(stream), C.c_uint32(dist_id), C.c_uint64(step),
                    C.c_uint64(draw), _p(out, C.c_uint32))
    return out


def alias_build(weights):
    w = np.ascontiguousarray(weights, dtype=np.float64)
    thresh = np.zeros(len(w), dtype=np.uint32)
    alias = np.zeros(len(w), dtype=np.uint32)
    _check(lib().nor_alias_build(_p(w, C.c_double), C.c_int64(len(w)), _p(thresh, C.c_uint32),
                                 _p(alias, C.c_uint32)), "alias_build")
    return thresh, alias


def sample_conform(table, num_keys, seed, dist_id, step, n, draw0=0):
    thresh, alias = table if table is not None else (None, None)
    out = np.zeros(n, dtype=np.uint32)
    _check(lib().nor_sample_conform(_p(thresh, C.c_uint32), _p(alias, C.c_uint32), C.c_int64(num_keys),
                                    C.c_uint64(seed), C.c_uint32(dist_id), C.c_uint64(step),
                                    C.c_uint64(draw0), C.c_int64(n), _p(out, C.c_uint32)), "sample_conform")
    return out


def sample_bounded(table, num_keys, seed, dist_id, step, n, U, G):
    thresh, alias = table if table is not None else (None, None)
    out = np.zeros(n, dtype=np.uint32)
    _check(lib().nor_sample_bounded(_p(thresh, C.c_uint32), _p(alias, C.c_uint32), C.c_int64(num_keys),
                                    C.c_uint64(seed), C.c_uint32(dist_id), C.c_uint64(step), C.c_int64(n),
                                    C.c_int32(U), C.c_int32(G), _p(out, C.c_uint32)), "sample_bounded")
    return out


def permute(x, P, seed, dist_id, epoch, pass_):
    return int(lib().nor_permute(C.c_uint64(x), C.c_uint64(P), C.c_uint64(seed), C.c_uint32(dist_id),
                                 C.c_uint64(epoch), C.c_uint64(pass_)))


def sample_longterm(table, num_keys, seed, dist_id, P, R, cursor, n):
    thresh, alias = table if table is not None else (None, None)
    out = np.zeros(n, dtype=np.uint32)
    _check(lib().nor_sample_longterm(_p(thresh, C.c_uint32), _p(alias, C.c_uint32), C.c_int64(num_keys),
                                     C.c_uint64(seed), C.c_uint32(dist_id), C.c_int64(P), C.c_int32(R),
                                     C.c_uint64(cursor), C.c_int64(n), _p(out, C.c_uint32)), "sample_longterm")
    return out


def postpone_within_handle(samples, resident_keys):
    """Sample reuse with postponing (Section 4.4), within the N samples of one handle: walking through the
    samples, one whose key is not local is moved to the end of the handle's samples and its key re-localised (it is
    local from then on); every sample is postponed at most once: those met a second time, towards the end, are used
    wherever their key is.  `resident_keys`: the keys that are local from the start (on one device: the declared hot
    keys, which a replication technique keeps local everywhere).  Pure Python, sample by sample, as the paper words it."""
    seq = [int(k) for k in samples]
    local = set(int(k) for k in resident_keys)
    postponed = [False] * len(seq)
    i = 0
    while i < len(seq):
        if seq[i] in local or postponed[i]:
            i += 1                                  # used here
            continue
        k = seq.pop(i)                              # not local: to the end of this handle's samples, once
        postponed.pop(i)
        seq.append(k)
        postponed.append(True)
        local.add(k)                                # its relocation has been requested
    return np.array(seq, dtype=np.uint32)


def sample_longterm_postponed(table, num_keys, seed, dist_id, P, R, cursor, n, resident_keys):
    """The n samples of a handle under sample reuse with postponing: the pool's sequence, postponed within the handle."""
    return postpone_within_handle(sample_longterm(table, num_keys, seed, dist_id, P, R, cursor, n), resident_keys)


def sample_nonconform(keys_a, keys_b, per_example, split, T, seed, dist_id, step, n):
    a, b = _u32(keys_a), _u32(keys_b)
    assert len(a) == len(b)
    out = np.zeros(n, dtype=np.uint32)
    _check(lib().nor_sample_nonconform(_p(a, C.c_uint32), _p(b, C.c_uint32), C.c_int64(len(a)),
                                       C.c_int32(per_example), C.c_int32(split), C.c_int32(T),
                                       C.c_uint64(seed), C.c_uint32(dist_id), C.c_uint64(step),
                                       C.c_int64(n), _p(out, C.c_uint32)), "sample_nonconform")
    return out


def distinct_keys(keys):
    k = _u32(keys)
    uniq = np.zeros(len(k), dtype=np.uint32)
    cnt = np.zeros(len(k), dtype=np.uint32)
    nu = lib().nor_distinct_keys(_p(k, C.c_uint32), C.c_int64(len(k)), _p(uniq, C.c_uint32), _p(cnt, C.c_uint32))
    if nu < 0:
        raise ValueError("oracle distinct_keys failed")
    return uniq[:nu].copy(), cnt[:nu].copy()


def pull(table, keys):
    t, k = _table(table), _u32(keys)
    out = np.zeros((len(k), t.shape[1]), dtype=np.float32)
    _check(lib().nor_pull(_p(t, C.c_float), C.c_int64(t.shape[0]), C.c_int32(t.shape[1]), _p(k, C.c_uint32),
                          C.c_int64(len(k)), _p(out, C.c_float)), "pull")
    return out


def push(table, dim, keys, updates):
    t, k = _table(table), _u32(keys)
    u = np.ascontiguousarray(updates, dtype=np.float32)
    assert u.shape == (len(k), t.shape[1])
    _check(lib().nor_push(_p(t, C.c_float), C.c_int64(t.shape[0]), C.c_int32(t.shape[1]), C.c_int32(dim),
                          _p(k, C.c_uint32), C.c_int64(len(k)), _p(u, C.c_float)), "push")


class Structure:
    """Distinct keys (ascending) and access counts of one table in one step."""

    def __init__(self, uniq, count):
        self.keys, self.counts = uniq, count


def _struct_bufs(n):
    return np.zeros(n + 1, dtype=np.uint32), np.zeros(n + 1, dtype=np.uint32), C.c_int64(0)


def step_sgns(In, Out, dim, center, context, negs, K, lr):
    """One step, in place on In and Out.  Returns (loss, Structure(In), Structure(Out))."""
    In, Out = _table(In), _table(Out)
    c, o, ng = _u32(center), _u32(context), _u32(negs)
    B = len(c)
    assert len(o) == B and len(ng) == B * K and In.shape[1] == Out.shape[1]
    loss = C.c_double(0.0)
    ui, ci, ni = _struct_bufs(B)
    uo, co, no = _struct_bufs(B * (K + 1))
    _check(lib().nor_step_sgns(_p(In, C.c_float), _p(Out, C.c_float), C.c_int64(In.shape[0]),
                               C.c_int64(Out.shape[0]), C.c_int32(In.shape[1]), C.c_int32(dim),
                               _p(c, C.c_uint32), _p(o, C.c_uint32), _p(ng, C.c_uint32), C.c_int64(B),
                               C.c_int32(K), C.c_float(lr), C.byref(loss),
                               _p(ui, C.c_uint32), _p(ci, C.c_uint32), C.byref(ni),
                               _p(uo, C.c_uint32), _p(co, C.c_uint32), C.byref(no)), "step_sgns")
    return loss.value, Structure(ui[:ni.value].copy(), ci[:ni.value].copy()), \
        Structure(uo[:no.value].copy(), co[:no.value].copy())


def _hot_flags(num_keys, hot_keys):
    """One byte per key: 1 for the keys of the hot set."""
    flags = np.zeros(num_keys, dtype=np.uint8)
    if hot_keys is not None and len(hot_keys):
        flags[np.asarray(hot_keys, dtype=np.int64)] = 1
    return flags


def step_sgns_clipped(In, Out, dim, center, context, negs, K, lr, hot_in, hot_out, factor, stats_in, stats_out):
    """step_sgns with the updates of the hot keys clipped at `factor` times their average norm so far.
    hot_*: key lists; stats_*: float64 arrays {sum of norms, number of norms}, updated in place.  Returns the loss."""
    In, Out = _table(In), _table(Out)
    c, o, ng = _u32(center), _u32(context), _u32(negs)
    B = len(c)
    assert len(o) == B and len(ng) == B * K and In.shape[1] == Out.shape[1]
    assert stats_in.dtype == np.float64 and stats_out.dtype == np.float64 and len(stats_in) == len(stats_out) == 2
    hi, ho = _hot_flags(In.shape[0], hot_in), _hot_flags(Out.shape[0], hot_out)
    loss = C.c_double(0.0)
    _check(lib().nor_step_sgns_clipped(_p(In, C.c_float), _p(Out, C.c_float), C.c_int64(In.shape[0]),
                                       C.c_int64(Out.shape[0]), C.c_int32(In.shape[1]), C.c_int32(dim),
                                       _p(c, C.c_uint32), _p(o, C.c_uint32), _p(ng, C.c_uint32), C.c_int64(B),
                                       C.c_int32(K), C.c_float(lr), C.byref(loss), _p(hi, C.c_uint8),
                                       _p(ho, C.c_uint8), C.c_double(factor), _p(stats_in, C.c_double),
                                       _p(stats_out, C.c_double)), "step_sgns_clipped")
    return loss.value


def loss_sgns(In, Out, dim, center, context, negs, K):
    In, Out = _table(In), _table(Out)
    c, o, ng = _u32(center), _u32(context), _u32(negs)
    return lib().nor_loss_sgns(_p(In, C.c_float), _p(Out, C.c_float), C.c_int32(In.shape[1]), C.c_int32(dim),
                               _p(c, C.c_uint32), _p(o, C.c_uint32), _p(ng, C.c_uint32), C.c_int64(len(c)),
                               C.c_int32(K))


def step_mf(W, H, dim, row, col, val, lr, l2):
    W, H = _table(W), _table(H)
    r, c = _u32(row), _u32(col)
    v = np.ascontiguousarray(val, dtype=np.float32)
    B = len(r)
    loss = C.c_double(0.0)
    uw, cw, nw = _struct_bufs(B)
    uh, ch, nh = _struct_bufs(B)
    _check(lib().nor_step_mf(_p(W, C.c_float), _p(H, C.c_float), C.c_int64(W.shape[0]), C.c_int64(H.shape[0]),
                             C.c_int32(W.shape[1]), C.c_int32(dim), _p(r, C.c_uint32), _p(c, C.c_uint32),
                             _p(v, C.c_float), C.c_int64(B), C.c_float(lr), C.c_float(l2), C.byref(loss),
                             _p(uw, C.c_uint32), _p(cw, C.c_uint32), C.byref(nw),
                             _p(uh, C.c_uint32), _p(ch, C.c_uint32), C.byref(nh)), "step_mf")
    return loss.value, Structure(uw[:nw.value].copy(), cw[:nw.value].copy()), \
        Structure(uh[:nh.value].copy(), ch[:nh.value].copy())


def step_mf_clipped(W, H, dim, row, col, val, lr, l2, hot_w, hot_h, factor, stats_w, stats_h):
    """step_mf with the updates of the hot rows / columns clipped (see step_sgns_clipped).  Returns the loss."""
    W, H = _table(W), _table(H)
    r, c = _u32(row), _u32(col)
    v = np.ascontiguousarray(val, dtype=np.float32)
    assert stats_w.dtype == np.float64 and stats_h.dtype == np.float64 and len(stats_w) == len(stats_h) == 2
    hw, hh = _hot_flags(W.shape[0], hot_w), _hot_flags(H.shape[0], hot_h)
    loss = C.c_double(0.0)
    _check(lib().nor_step_mf_clipped(_p(W, C.c_float), _p(H, C.c_float), C.c_int64(W.shape[0]),
                                     C.c_int64(H.shape[0]), C.c_int32(W.shape[1]), C.c_int32(dim),
                                     _p(r, C.c_uint32), _p(c, C.c_uint32), _p(v, C.c_float), C.c_int64(len(r)),
                                     C.c_float(lr), C.c_float(l2), C.byref(loss), _p(hw, C.c_uint8),
                                     _p(hh, C.c_uint8), C.c_double(factor), _p(stats_w, C.c_double),
                                     _p(stats_h, C.c_double)), "step_mf_clipped")
    return loss.value


def loss_mf(W, H, dim, row, col, val, l2):
    W, H = _table(W), _table(H)
    r, c = _u32(row), _u32(col)
    v = np.ascontiguousarray(val, dtype=np.float32)
    return lib().nor_loss_mf(_p(W, C.c_float), _p(H, C.c_float), C.c_int32(W.shape[1]), C.c_int32(dim),
                             _p(r, C.c_uint32), _p(c, C.c_uint32), _p(v, C.c_float), C.c_int64(len(r)),
                             C.c_float(l2))


def step_kge(E, GE, R, GR, dim, subj, rel, obj, negs, nh, nt, lr, eps):
    E, GE, R, GR = _table(E), _table(GE), _table(R), _table(GR)
    s, r, o, ng = _u32(subj), _u32(rel), _u32(obj), _u32(negs)
    B = len(s)
    assert len(ng) == B * (nh + nt)
    loss = C.c_double(0.0)
    ue, ce, ne = _struct_bufs(B * (2 + nh + nt))
    ur, cr, nr = _struct_bufs(B)
    _check(lib().nor_step_kge(_p(E, C.c_float), _p(GE, C.c_float), _p(R, C.c_float), _p(GR, C.c_float),
                              C.c_int64(E.shape[0]), C.c_int64(R.shape[0]), C.c_int32(E.shape[1]),
                              C.c_int32(dim), _p(s, C.c_uint32), _p(r, C.c_uint32), _p(o, C.c_uint32),
                              _p(ng, C.c_uint32), C.c_int64(B), C.c_int32(nh), C.c_int32(nt),
                              C.c_float(lr), C.c_float(eps), C.byref(loss),
                              _p(ue, C.c_uint32), _p(ce, C.c_uint32), C.byref(ne),
                              _p(ur, C.c_uint32), _p(cr, C.c_uint32), C.byref(nr)), "step_kge")
    return loss.value, Structure(ue[:ne.value].copy(), ce[:ne.value].copy()), \
        Structure(ur[:nr.value].copy(), cr[:nr.value].copy())


def loss_kge(E, R, dim, subj, rel, obj, negs, nh, nt):
    E, R = _table(E), _table(R)
    s, r, o, ng = _u32(subj), _u32(rel), _u32(obj), _u32(negs)
    return lib().nor_loss_kge(_p(E, C.c_float), _p(R, C.c_float), C.c_int32(E.shape[1]), C.c_int32(dim),
                              _p(s, C.c_uint32), _p(r, C.c_uint32), _p(o, C.c_uint32), _p(ng, C.c_uint32),
                              C.c_int64(len(s)), C.c_int32(nh), C.c_int32(nt))


def complex_score(s_row, r_row, o_row, dim):
    """Score of one triple; rows are stored rows (real parts at 0, imaginary parts at len/2)."""
    s = np.ascontiguousarray(s_row, dtype=np.float32)
    r = np.ascontiguousarray(r_row, dtype=np.float32)
    o = np.ascontiguousarray(o_row, dtype=np.float32)
    assert len(s) == len(r) == len(o)
    return lib().nor_complex_score(_p(s, C.c_float), _p(r, C.c_float), _p(o, C.c_float), C.c_int32(len(s)),
                                   C.c_int32(dim))
