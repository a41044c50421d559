"""Pins of the oracle's steps with stale replicas of the hot keys (oracle/replicas.py; Section 3.2 of the paper:
replicas of hot-spot keys, updated locally and synchronised periodically by exchanging accumulated updates)."""
import numpy as np

from oracle import oracle as orc
from oracle import replicas as rep
from paper_2104_00501_amd import workloads as wl


def test_remapping_against_a_loop():
    V, R, B, K = 50, 3, 11, 2
    hot = [7, 0, 31]
    slot = rep.hot_slots(V, hot)
    assert list(slot[[7, 0, 31]]) == [0, 1, 2] and (slot >= 0).sum() == 3
    rng = np.random.default_rng(1)
    keys = rng.integers(0, V, B * K)
    keys[::4] = 31
    got = rep.remap_keys(keys, np.repeat(np.arange(B), K), B, V, slot, R)
    for p, k in enumerate(keys):
        e = p // K
        part = (e * R) // B                      # contiguous parts: 0,0,0,0 | 1,1,1,1 | 2,2,2 for B = 11
        want = V + part * 3 + hot.index(k) if k in hot else k
        assert got[p] == want
    assert list(rep.part_of(np.arange(11), 11, 3)) == [0, 0, 0, 0, 1, 1, 1, 1, 2, 2, 2]


def test_hand_worked_two_replica_example():
    # Factorisation with one-number rows, lr = 1/4, no regulariser; column 0 is hot with two replicas.
    # Part 0 = cell (row 0, col 0, x = 1), part 1 = cell (row 1, col 0, x = 0); w = (1, 2), h = 1/2.
    # Step 1: part 0: err = 1/2, w0 = 1 + 1/8 = 1.125, its replica h = 1/2 + 1/4 = 0.75;
    #         part 1: err = -1, w1 = 2 - 1/4 = 1.75, its replica h = 1/2 - 1 = -0.5.
    # Step 2 (no synchronisation in between: each part still sees only its own replica):
    #         part 0: err = 1 - 1.125 * 0.75 = 0.15625, w0 = 1.18359375, h = 0.75 + 0.087890625 = 0.837890625;
    #         part 1: err = 0 + 1.75 * 0.5 = 0.875, w1 = 1.75 - 0.21875 = 1.53125, h = -0.5 + 0.765625 = 0.265625.
    # Synchronisation: h = 1/2 + (0.837890625 - 1/2) + (0.265625 - 1/2) = 0.603515625 everywhere.
    W = np.array([[1.0], [2.0]], dtype=np.float32)
    H = np.array([[0.5], [9.0]], dtype=np.float32)
    W_ext, H_ext = rep.extend_table(W, [], 2), rep.extend_table(H, [0], 2)
    assert H_ext.shape == (4, 1)
    rows, cols, vals = np.array([0, 1], dtype=np.uint32), np.array([0, 0], dtype=np.uint32), np.array([1, 0], dtype=np.float32)
    rep.step_mf_replicated(W_ext, H_ext, 1, rows, cols, vals, 0.25, 0.0, 2, 2, [], [0], 2)
    assert list(W_ext[:, 0]) == [1.125, 1.75] and list(H_ext[:, 0]) == [0.5, 9.0, 0.75, -0.5]
    rep.step_mf_replicated(W_ext, H_ext, 1, rows, cols, vals, 0.25, 0.0, 2, 2, [], [0], 2)
    assert list(W_ext[:, 0]) == [1.18359375, 1.53125] and list(H_ext[:, 0]) == [0.5, 9.0, 0.837890625, 0.265625]
    rep.sync_replicas(H_ext, 2, [0], 2, 1)
    assert list(H_ext[:, 0]) == [0.603515625, 9.0, 0.603515625, 0.603515625]
    rep.sync_replicas(H_ext, 2, [0], 2, 1)                       # nothing accumulated: nothing changes
    assert list(H_ext[:, 0]) == [0.603515625, 9.0, 0.603515625, 0.603515625]
    # the plain steps see the other part's update at once: a different value
    Wp, Hp = W.copy(), H.copy()
    for _ in range(2):
        orc.step_mf(Wp, Hp, 1, rows, cols, vals, 0.25, 0.0)
    assert Hp[0, 0] != np.float32(0.603515625)


def _sgns_case(V, d, B, K, seed):
    toks = wl.zipf_stream(V, 1.1, B // 4 + 8, seed)
    c, o = wl.window_pairs(toks, 2, 0, B)
    In = wl.uniform_table(V, d, -0.5, 0.5, seed + 1)
    Out = wl.uniform_table(V, d, -0.5, 0.5, seed + 2)
    negs = wl.zipf_stream(V, 0.8, len(c) * K, seed + 3)
    return c, o, negs, In, Out


def test_one_replica_is_the_plain_step_bit_for_bit():
    # with one part the replica is simply where the hot key lives between synchronisations
    V, d, K, steps = 60, 8, 2, 4
    c, o, negs, In, Out = _sgns_case(V, d, 40, K, 3)
    hot_in, hot_out = [0, 1, 5], [0, 2]
    Ie, Oe = rep.extend_table(In, hot_in, 1), rep.extend_table(Out, hot_out, 1)
    Ip, Op = In.copy(), Out.copy()
    for t in range(steps):
        la = rep.step_sgns_replicated(Ie, Oe, d, c, o, negs, K, 0.05, V, V, hot_in, hot_out, 1)
        lb = orc.step_sgns(Ip, Op, d, c, o, negs, K, 0.05)[0]
        assert la == lb
        assert np.array_equal(Ie[V:], Ip[hot_in]) and np.array_equal(Oe[V:], Op[hot_out])     # replicas = plain values
        cold = np.setdiff1d(np.arange(V), hot_in)
        assert np.array_equal(Ie[cold], Ip[cold])
        assert np.array_equal(Ie[hot_in], In[hot_in])            # the base waits for the synchronisation
    rep.sync_replicas(Ie, V, hot_in, 1, d)
    rep.sync_replicas(Oe, V, hot_out, 1, d)
    assert np.array_equal(Ie[:V], Ip) and np.array_equal(Oe[:V], Op)


def test_no_hot_key_in_the_batch_is_the_plain_step():
    V, d, K = 60, 8, 2
    c, o, negs, In, Out = _sgns_case(V, d, 40, K, 4)
    hot = [k for k in range(V) if k not in set(c) | set(o) | set(negs)][:3]
    assert len(hot) == 3
    Ie, Oe = rep.extend_table(In, hot, 4), rep.extend_table(Out, hot, 4)
    rep.step_sgns_replicated(Ie, Oe, d, c, o, negs, K, 0.05, V, V, hot, hot, 4)
    Ip, Op = In.copy(), Out.copy()
    orc.step_sgns(Ip, Op, d, c, o, negs, K, 0.05)
    assert np.array_equal(Ie[:V], Ip) and np.array_equal(Oe[:V], Op)
    assert np.array_equal(Ie[V:], np.concatenate([In[hot]] * 4))


def test_a_step_is_the_plain_step_of_each_part_on_its_own_view():
    # Part r computes as if the hot rows were its replicas and only its own examples existed; rows that are not
    # hot collect every part's update.  Replica rows: bit for bit; shared rows: to rounding (one rounding of the
    # whole sum against one per part).
    V, d, K, R, B = 80, 8, 3, 4, 64
    c, o, negs, In, Out = _sgns_case(V, d, B, K, 5)
    B = len(c)
    hot_in, hot_out = [0, 1, 2, 3], [0, 1, 4]
    Ie, Oe = rep.extend_table(In, hot_in, R), rep.extend_table(Out, hot_out, R)
    rng = np.random.default_rng(0)
    Ie[V:] += rng.normal(0, 0.05, Ie[V:].shape).astype(np.float32)        # replicas that have drifted apart
    Oe[V:] += rng.normal(0, 0.05, Oe[V:].shape).astype(np.float32)
    I0, O0 = Ie.copy(), Oe.copy()
    rep.step_sgns_replicated(Ie, Oe, d, c, o, negs, K, 0.05, V, V, hot_in, hot_out, R)
    sum_in, sum_out = np.zeros(In.shape), np.zeros(Out.shape)
    parts = rep.part_of(np.arange(B), B, R)
    for r in range(R):
        sel = parts == r
        Iv, Ov = I0[:V].copy(), O0[:V].copy()
        Iv[hot_in] = I0[V + r * len(hot_in):V + (r + 1) * len(hot_in)]
        Ov[hot_out] = O0[V + r * len(hot_out):V + (r + 1) * len(hot_out)]
        Ia, Oa = Iv.copy(), Ov.copy()
        orc.step_sgns(Ia, Oa, d, c[sel], o[sel], negs.reshape(B, K)[sel].ravel(), K, 0.05)
        assert np.array_equal(Ia[hot_in], Ie[V + r * len(hot_in):V + (r + 1) * len(hot_in)])
        assert np.array_equal(Oa[hot_out], Oe[V + r * len(hot_out):V + (r + 1) * len(hot_out)])
        sum_in += Ia.astype(np.float64) - Iv
        sum_out += Oa.astype(np.float64) - Ov
    cold_in, cold_out = np.setdiff1d(np.arange(V), hot_in), np.setdiff1d(np.arange(V), hot_out)
    assert np.allclose(Ie[cold_in], I0[cold_in] + sum_in[cold_in], rtol=0, atol=2e-7)
    assert np.allclose(Oe[cold_out], O0[cold_out] + sum_out[cold_out], rtol=0, atol=2e-7)
    assert np.array_equal(Ie[hot_in], I0[hot_in]) and np.array_equal(Oe[hot_out], O0[hot_out])   # bases untouched


def test_synchronising_after_every_step_is_the_plain_step_to_rounding():
    V, d, K, R = 80, 8, 3, 8
    c, o, negs, In, Out = _sgns_case(V, d, 64, K, 6)
    hot = [0, 1, 2, 3, 4]
    Ie, Oe = rep.extend_table(In, hot, R), rep.extend_table(Out, hot, R)
    Ip, Op = In.copy(), Out.copy()
    for _ in range(3):
        rep.step_sgns_replicated(Ie, Oe, d, c, o, negs, K, 0.05, V, V, hot, hot, R)
        rep.sync_replicas(Ie, V, hot, R, d)
        rep.sync_replicas(Oe, V, hot, R, d)
        orc.step_sgns(Ip, Op, d, c, o, negs, K, 0.05)
        for r in range(R):                                   # every replica holds the synchronised value
            assert np.array_equal(Ie[V + r * 5:V + (r + 1) * 5], Ie[hot])
    assert np.allclose(Ie[:V], Ip, rtol=0, atol=1e-6) and np.allclose(Oe[:V], Op, rtol=0, atol=1e-6)
    assert not np.array_equal(Ie[:V], In)


def test_synchronisation_adds_the_replicas_accumulated_updates():
    # dyadic numbers: base 1, replicas 1.5, 0.75, 1 -> 1 + 0.5 - 0.25 + 0 = 1.25; lanes beyond dim are left alone
    ext = np.array([[1.0, 7.0], [3.0, 7.0], [1.5, 7.0], [0.75, 7.0], [1.0, 7.0]], dtype=np.float32)
    rep.sync_replicas(ext, 2, [0], 3, 1)
    assert list(ext[:, 0]) == [1.25, 3.0, 1.25, 1.25, 1.25] and list(ext[:, 1]) == [7.0] * 5
