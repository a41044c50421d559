"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, rejects bad arguments, and builds the same alias table as the oracle bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2104_00501_amd import binding as nb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_entry_point_is_exported():
    header = open(os.path.join(ROOT, "include", "nups.h")).read()
    declared = set(re.findall(r"\b(nups_[a-z_]+)\s*\(", header))
    declared -= {"nups_status", "nups_scheme", "nups_task"}
    assert declared == set(nb.EXPORTS)
    lib = nb.lib()
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("seed,V", [(0, 1), (1, 2), (2, 33), (3, 1000), (4, 50000)])
def test_alias_table_equals_the_oracles(seed, V):
    rng = np.random.default_rng(seed)
    w = rng.random(V) ** 4
    w[rng.random(V) < 0.3] = 0
    w[0] = 0.5
    t1, a1 = nb.nups_build_alias_table(w)
    t2, a2 = orc.alias_build(w)
    assert np.array_equal(t1, t2) and np.array_equal(a1, a2)


def test_alias_table_zipf_weights_equal_the_oracles():
    w = (np.arange(1, 200001, dtype=np.float64) ** -1.0 * 1e9) ** 0.75
    t1, a1 = nb.nups_build_alias_table(w)
    t2, a2 = orc.alias_build(w)
    assert np.array_equal(t1, t2) and np.array_equal(a1, a2)


def test_alias_table_rejects_bad_weights():
    for bad in ([0.0, 0.0], [1.0, -1.0], [1.0, float("nan")], [float("inf"), 1.0]):
        with pytest.raises(nb.NupsError) as e:
            nb.nups_build_alias_table(np.array(bad))
        assert e.value.status == nb.NUPS_ERR_ARG
    assert "weights" in nb.nups_last_error()


def test_init_rejects_bad_shapes_before_touching_the_device():
    lib = nb.lib()
    ctx = C.c_void_p(None)
    ptrs = (C.c_void_p * 1)(0x1000)
    def call(nk, dim, stride, n=1, tables=ptrs):
        return lib.nups_init(C.byref(ctx), C.c_int(n), tables, (C.c_int64 * 1)(nk), (C.c_int32 * 1)(dim),
                             (C.c_int32 * 1)(stride), None)
    assert call(10, 100, 64) == nb.NUPS_ERR_ARG          # dim > row_stride
    assert call(10, 100, 100) == nb.NUPS_ERR_ARG         # stride not a multiple of 64
    assert call(10, 100, 2048) == nb.NUPS_ERR_ARG        # stride too large
    assert call(10, 100, 448) == nb.NUPS_ERR_ARG         # a multiple of 64 outside the supported set
    assert call(10, 100, 960) == nb.NUPS_ERR_ARG
    assert call(0, 100, 128) == nb.NUPS_ERR_ARG          # no keys
    assert call(10, 0, 128) == nb.NUPS_ERR_ARG
    assert call(10, 100, 128, n=0) == nb.NUPS_ERR_ARG
    assert call(10, 100, 128, n=5) == nb.NUPS_ERR_ARG
    assert call(10, 100, 128, tables=(C.c_void_p * 1)(None)) == nb.NUPS_ERR_ARG
    assert lib.nups_init(None, 1, ptrs, None, None, None, None) == nb.NUPS_ERR_ARG
    assert ctx.value is None


def test_null_objects_are_rejected():
    lib = nb.lib()
    assert lib.nups_destroy(None) == nb.NUPS_ERR_ARG
    assert lib.nups_step(None, None, None) == nb.NUPS_ERR_ARG
    assert lib.nups_pull(None, 0, None, 0, None) == nb.NUPS_ERR_ARG
    assert lib.nups_release_sample(None) == nb.NUPS_ERR_ARG
    assert lib.nups_pull_sample(None, C.c_int64(1), None, None) == nb.NUPS_ERR_ARG
    assert lib.nups_prepare_sample(None, C.c_int64(1), C.c_uint64(0), C.byref(C.c_void_p())) == nb.NUPS_ERR_ARG
    assert lib.nups_check(None) == nb.NUPS_ERR_ARG
    assert lib.nups_set_postponing(None, C.c_int(1)) == nb.NUPS_ERR_ARG
    assert nb.nups_phase_name(nb.NUPS_PHASE_GRAD) == "grad" and nb.nups_phase_name(99) == ""


def test_hot_key_heuristic_against_brute_force_and_the_zipf_closed_form():
    # Section 5.1, untuned configuration: hot = access frequency above 100 x the mean access frequency
    rng = np.random.default_rng(4)
    f = rng.pareto(0.7, 5000)
    f[[10, 20, 30]] = f.max() * 2                          # ties among the most frequent keys
    hot = nb.nups_select_hot_keys(f, 20.0)
    brute = [k for k in range(len(f)) if f[k] > 20.0 * f.sum() / len(f)]
    assert sorted(hot.tolist()) == brute and len(hot) > 5
    assert hot[:3].tolist() == [10, 20, 30]                # most frequent first, ties by key
    assert np.all(np.diff(f[hot]) <= 0)
    # Zipf(1) over V keys: p_k = 1 / (k H_V), mean 1 / V: key of rank k is hot iff k < V / (100 H_V)
    V = 1_000_000
    p = 1.0 / np.arange(1, V + 1)
    H_V = p.sum()
    hot = nb.nups_select_hot_keys(p / H_V)
    assert len(hot) == int(np.ceil(V / (100.0 * H_V))) - 1 and np.array_equal(hot, np.arange(len(hot)))
    assert len(nb.nups_select_hot_keys(np.ones(1000))) == 0          # uniform access: nothing is hot
    for bad in ([1.0, -1.0], [float("nan"), 1.0]):
        with pytest.raises(nb.NupsError) as e:
            nb.nups_select_hot_keys(np.array(bad))
        assert e.value.status == nb.NUPS_ERR_ARG
    with pytest.raises(nb.NupsError):
        nb.nups_select_hot_keys(np.ones(4), 0.0)
