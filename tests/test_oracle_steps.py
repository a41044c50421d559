"""Pins for the oracle's step arithmetic: finite differences of separately written
loss functions, closed forms, reductions to simpler models, batching invariants
(CPU only)."""
import numpy as np
import pytest

from oracle import oracle as orc

H = 2.0 ** -7


def _quantised(rng, shape, stride, scale=1.0):
    """fp32 table whose entries are multiples of 2^-10 so that +-H and +-2H are exact."""
    t = np.zeros((shape[0], stride), dtype=np.float32)
    t[:, :shape[1]] = np.round(rng.uniform(-scale, scale, shape) * 1024) / 1024
    return t


def _fd(loss, table, dim, cols=None):
    """Fourth-order central differences of loss() w.r.t. the lanes `cols` (default: first dim) of every row."""
    cols = list(range(dim)) if cols is None else list(cols)
    g = np.zeros((table.shape[0], len(cols)))
    for r in range(table.shape[0]):
        for gi, c in enumerate(cols):
            x0 = table[r, c]
            f = []
            for k in (1, -1, 2, -2):
                table[r, c] = np.float32(x0 + k * H)
                f.append(loss())
            table[r, c] = x0
            g[r, gi] = (8 * (f[0] - f[1]) - (f[2] - f[3])) / (12 * H)
    return g


# ----------------------------------------------------------------------------- SGNS
def _sgns_case(seed, V=6, d=3, B=7, K=2, stride=64):
    rng = np.random.default_rng(seed)
    In, Out = _quantised(rng, (V, d), stride), _quantised(rng, (V, d), stride)
    c = rng.integers(0, V, B).astype(np.uint32)
    o = rng.integers(0, V, B).astype(np.uint32)
    ng = rng.integers(0, V, B * K).astype(np.uint32)
    return In, Out, c, o, ng


@pytest.mark.parametrize("seed,K", [(0, 2), (1, 0), (2, 5), (3, 1)])
def test_sgns_step_is_a_gradient_step_on_the_summed_batch_loss(seed, K):
    d = 3
    In, Out, c, o, ng = _sgns_case(seed, K=K)
    gi = _fd(lambda: orc.loss_sgns(In, Out, d, c, o, ng, K), In, d)
    go = _fd(lambda: orc.loss_sgns(In, Out, d, c, o, ng, K), Out, d)
    In1, Out1 = In.copy(), Out.copy()
    lr = 0.5
    loss, s_in, s_out = orc.step_sgns(In1, Out1, d, c, o, ng, K, lr)
    assert abs(loss - orc.loss_sgns(In, Out, d, c, o, ng, K)) < 1e-12 * max(1, abs(loss))
    # duplicates in the batch (V=6, B=7 forces them) are summed, against the pre-step snapshot
    assert np.max(np.abs((In[:, :d] - In1[:, :d]) / lr - gi)) < 3e-7
    assert np.max(np.abs((Out[:, :d] - Out1[:, :d]) / lr - go)) < 3e-7
    assert np.all(In1[:, d:] == 0) and np.all(Out1[:, d:] == 0)             # padding untouched
    assert np.array_equal(s_in.keys, np.unique(c))
    assert np.array_equal(s_in.counts, np.unique(c, return_counts=True)[1])
    allo = np.concatenate([o, ng])
    assert np.array_equal(s_out.keys, np.unique(allo))
    assert np.array_equal(s_out.counts, np.unique(allo, return_counts=True)[1])
    assert s_out.counts.sum() == len(c) * (K + 1)


def test_sgns_without_negatives_is_logistic_regression_on_one_dot_product():
    d = 4
    v = np.zeros((1, 64), np.float32); u = np.zeros((1, 64), np.float32)
    v[0, :d] = [0.5, -0.25, 1.0, 0.125]; u[0, :d] = [-1.0, 0.5, 0.25, 2.0]
    z = float(np.dot(v[0, :d].astype(np.float64), u[0, :d]))
    g = 1.0 / (1.0 + np.exp(-z)) - 1.0
    v1, u1 = v.copy(), u.copy()
    loss, _, _ = orc.step_sgns(v1, u1, d, [0], [0], [], 0, 0.25)
    assert abs(loss - np.log1p(np.exp(-z))) < 1e-14
    assert np.allclose(v1[0, :d], v[0, :d] - 0.25 * g * u[0, :d], rtol=0, atol=1e-7)
    assert np.allclose(u1[0, :d], u[0, :d] - 0.25 * g * v[0, :d], rtol=0, atol=1e-7)


def test_sgns_negative_sign_and_table_roles():
    # one pair, one negative, orthogonal rows: z = 0 for both, so g_pos = -1/2 and g_neg = +1/2
    d = 2
    In = np.zeros((3, 64), np.float32); Out = np.zeros((3, 64), np.float32)
    In[0, :d] = [1, 0]; Out[1, :d] = [0, 1]; Out[2, :d] = [0, -1]
    loss, _, _ = orc.step_sgns(In, Out, d, [0], [1], [2], 1, 1.0)
    assert abs(loss - 2 * np.log(2)) < 1e-14
    assert np.allclose(In[0, :d], [1, 0 - (-0.5 * 1 + 0.5 * -1)])          # v - (g_pos u_pos + g_neg u_neg)
    assert np.allclose(Out[1, :d], [0.5, 1]) and np.allclose(Out[2, :d], [-0.5, -1])
    assert np.all(In[1:] == 0) and np.all(Out[0] == 0)                      # negatives never touch the input table


def test_sgns_batch_with_distinct_keys_equals_independent_single_steps():
    d, B, K, V = 5, 6, 2, 64
    rng = np.random.default_rng(4)
    In, Out = _quantised(rng, (V, d), 64), _quantised(rng, (V, d), 64)
    perm = rng.permutation(V).astype(np.uint32)
    c, rest = perm[:B], rng.permutation(V)[:B * (K + 1)].astype(np.uint32)
    o, ng = rest[:B], rest[B:]
    A, Bt = In.copy(), Out.copy()
    orc.step_sgns(A, Bt, d, c, o, ng, K, 0.1)
    A2, B2 = In.copy(), Out.copy()
    for e in range(B):
        orc.step_sgns(A2, B2, d, c[e:e + 1], o[e:e + 1], ng[e * K:(e + 1) * K], K, 0.1)
    assert np.array_equal(A, A2) and np.array_equal(Bt, B2)


def test_sgns_delta_is_additive_over_a_split_of_the_batch_and_order_free():
    d, V, B, K = 4, 5, 12, 3
    In, Out, c, o, ng = _sgns_case(9, V=V, d=d, B=B, K=K)
    full_i, full_o = In.copy(), Out.copy()
    orc.step_sgns(full_i, full_o, d, c, o, ng, K, 0.25)
    di, do = np.zeros_like(In, dtype=np.float64), np.zeros_like(Out, dtype=np.float64)
    for lo, hi in ((0, 5), (5, 12)):
        a, b = In.copy(), Out.copy()
        orc.step_sgns(a, b, d, c[lo:hi], o[lo:hi], ng[lo * K:hi * K], K, 0.25)
        di += a.astype(np.float64) - In; do += b.astype(np.float64) - Out
    assert np.max(np.abs(full_i - In - di)) < 4e-7 and np.max(np.abs(full_o - Out - do)) < 4e-7
    p = np.random.default_rng(1).permutation(B)
    a, b = In.copy(), Out.copy()
    orc.step_sgns(a, b, d, c[p], o[p], ng.reshape(B, K)[p].ravel(), K, 0.25)
    assert np.max(np.abs(a - full_i)) < 2e-7 and np.max(np.abs(b - full_o)) < 2e-7


def test_step_rejects_keys_out_of_range():
    In, Out, c, o, ng = _sgns_case(0)
    with pytest.raises(ValueError):
        orc.step_sgns(In, Out, 3, c, o, np.full_like(ng, 6), 2, 0.1)


# ----------------------------------------------------------------------------- MF
@pytest.mark.parametrize("seed,l2", [(0, 0.0), (1, 0.01), (2, 0.5)])
def test_mf_step_is_a_gradient_step_on_the_summed_batch_loss(seed, l2):
    rng = np.random.default_rng(seed)
    d, nr, nc, B = 3, 4, 3, 9
    W, Hh = _quantised(rng, (nr, d), 64), _quantised(rng, (nc, d), 64)
    r = rng.integers(0, nr, B).astype(np.uint32); c = rng.integers(0, nc, B).astype(np.uint32)
    x = (np.round(rng.normal(size=B) * 256) / 256).astype(np.float32)
    gw = _fd(lambda: orc.loss_mf(W, Hh, d, r, c, x, l2), W, d)
    gh = _fd(lambda: orc.loss_mf(W, Hh, d, r, c, x, l2), Hh, d)
    W1, H1 = W.copy(), Hh.copy()
    lr = 0.125
    loss, sw, sh = orc.step_mf(W1, H1, d, r, c, x, lr, l2)
    assert abs(loss - orc.loss_mf(W, Hh, d, r, c, x, l2)) < 1e-12 * max(1, abs(loss))
    assert np.max(np.abs((W[:, :d] - W1[:, :d]) / lr - gw)) < 2e-6
    assert np.max(np.abs((Hh[:, :d] - H1[:, :d]) / lr - gh)) < 2e-6
    assert np.array_equal(sw.keys, np.unique(r)) and np.array_equal(sh.counts, np.unique(c, return_counts=True)[1])


def test_mf_single_cell_rank_one_is_scalar_least_squares():
    W = np.zeros((1, 64), np.float32); Hh = np.zeros((1, 64), np.float32)
    W[0, 0], Hh[0, 0] = 0.5, -2.0
    x, lr = 3.0, 0.125
    err = x - 0.5 * -2.0
    loss, _, _ = orc.step_mf(W, Hh, 1, [0], [0], np.array([x], np.float32), lr, 0.0)
    assert loss == err * err
    assert W[0, 0] == np.float32(0.5 + lr * 2 * err * -2.0) and Hh[0, 0] == np.float32(-2.0 + lr * 2 * err * 0.5)


def test_mf_regulariser_counts_once_per_cell_occurrence():
    # zero residual: only the L2 term acts; a row seen 3 times shrinks by 3 * 2 * l2 * lr
    W = np.zeros((2, 64), np.float32); Hh = np.zeros((2, 64), np.float32)
    W[0, :2] = [1, 0]; Hh[0, :2] = [1, 0]; Hh[1, :2] = [1, 1]
    x = np.array([1, 1, 1], np.float32)
    orc.step_mf(W, Hh, 2, [0, 0, 0], [0, 1, 1], x, 0.5, 0.25)
    assert np.allclose(W[0, :2], [1 - 0.5 * 3 * 2 * 0.25 * 1, 0])
    assert np.allclose(Hh[1, :2], [1 - 0.5 * 2 * 2 * 0.25, 1 - 0.5 * 2 * 2 * 0.25])


# ----------------------------------------------------------------------------- KGE
def _ccols(d, stride=64):
    """Lanes of a stored complex row: d/2 real parts from 0, d/2 imaginary parts from stride/2."""
    return list(range(d // 2)) + list(range(stride // 2, stride // 2 + d // 2))


def _rows(rng, n, d, stride=64):
    t = np.zeros((n, stride), dtype=np.float32)
    t[:, _ccols(d, stride)] = _quantised(rng, (n, d), d)
    return t


def test_complex_score_is_real_part_of_trilinear_product_with_conjugated_object():
    rng = np.random.default_rng(0)
    d = 10
    s, r, o = (_rows(rng, 1, d)[0] for _ in range(3))
    cs, cr, co = (x[:5].astype(np.float64) + 1j * x[32:37] for x in (s, r, o))
    assert abs(orc.complex_score(s, r, o, d) - np.sum(cs * cr * np.conj(co)).real) < 1e-14


def test_complex_score_special_cases():
    rng = np.random.default_rng(1)
    d = 8
    s, r, o = (_rows(rng, 1, d)[0] for _ in range(3))
    z = lambda x: np.concatenate([x[:32], np.zeros(32, np.float32)])
    # all imaginary parts zero: DistMult, a plain trilinear product
    assert abs(orc.complex_score(z(s), z(r), z(o), d) - np.sum(s[:4].astype(np.float64) * r[:4] * o[:4])) < 1e-14
    # relation = 1: the Hermitian inner product's real part, i.e. the dot product of the stored rows
    one = np.zeros(64, np.float32); one[:4] = 1
    assert abs(orc.complex_score(s, one, o, d) - np.dot(s.astype(np.float64), o)) < 1e-14
    # real relation: symmetric in subject and object; purely imaginary relation: antisymmetric
    rr = z(r); ri = r.copy(); ri[:32] = 0
    assert abs(orc.complex_score(s, rr, o, d) - orc.complex_score(o, rr, s, d)) < 1e-14
    assert abs(orc.complex_score(s, ri, o, d) + orc.complex_score(o, ri, s, d)) < 1e-14


@pytest.mark.parametrize("seed,nh,nt", [(0, 1, 1), (1, 2, 0), (2, 0, 3), (3, 0, 0)])
def test_kge_step_follows_the_gradient_of_the_logistic_loss_through_adagrad(seed, nh, nt):
    rng = np.random.default_rng(seed)
    d, ne, nr, B = 4, 5, 2, 4
    E, R = _rows(rng, ne, d), _rows(rng, nr, d)
    s = rng.integers(0, ne, B).astype(np.uint32); o = rng.integers(0, ne, B).astype(np.uint32)
    r = rng.integers(0, nr, B).astype(np.uint32)
    ng = rng.integers(0, ne, B * (nh + nt)).astype(np.uint32)
    cc = _ccols(d)
    ge = _fd(lambda: orc.loss_kge(E, R, d, s, r, o, ng, nh, nt), E, d, cc)
    gr = _fd(lambda: orc.loss_kge(E, R, d, s, r, o, ng, nh, nt), R, d, cc)
    E1, R1 = E.copy(), R.copy()
    GE, GR = np.zeros_like(E), np.zeros_like(R)
    lr, eps = 0.125, 1e-10
    loss, se, sr = orc.step_kge(E1, GE, R1, GR, d, s, r, o, ng, nh, nt, lr, eps)
    assert abs(loss - orc.loss_kge(E, R, d, s, r, o, ng, nh, nt)) < 1e-12 * max(1, abs(loss))
    # from zero state the accumulator is the squared summed gradient and the move is lr * sign
    pad = np.setdiff1d(np.arange(64), cc)
    for tab, tab1, G, g in ((E, E1, GE, ge), (R, R1, GR, gr)):
        assert np.max(np.abs(G[:, cc] - g * g)) < 1e-5
        assert np.max(np.abs(np.sqrt(G[:, cc]) * np.sign(tab[:, cc] - tab1[:, cc]) - g)) < 2e-6
        moved = np.abs(g) > 1e-3
        assert np.allclose(np.abs(tab[:, cc] - tab1[:, cc])[moved], lr, rtol=1e-5)
        assert np.all(tab1[:, pad] == 0) and np.all(G[:, pad] == 0)
    allk = np.concatenate([s, o, ng])
    assert np.array_equal(se.keys, np.unique(allk)) and se.counts.sum() == B * (2 + nh + nt)
    assert np.array_equal(sr.keys, np.unique(r)) and np.array_equal(sr.counts, np.unique(r, return_counts=True)[1])
    untouched = np.setdiff1d(np.arange(ne), se.keys)
    assert np.array_equal(E1[untouched], E[untouched]) and np.all(GE[untouched] == 0)


def test_kge_negative_roles_subject_then_object():
    # scores pick out which slot a negative replaced: with relation (1, 0) the score is <s, o>
    d = 2
    E = np.zeros((4, 64), np.float32); R = np.zeros((1, 64), np.float32)
    R[0, 0] = 1.0
    E[0, :2] = [1, 0]; E[1, :2] = [2, 0]; E[2, :2] = [4, 0]; E[3, :2] = [8, 0]
    sp = lambda x: np.log1p(np.exp(x))
    # triple (0, 0, 1); nh=1 negative subject 2 -> score <E2,E1>=8; nt=1 negative object 3 -> <E0,E3>=8
    l_ht = orc.loss_kge(E, R, d, [0], [0], [1], [2, 3], 1, 1)
    assert abs(l_ht - (sp(-2.0) + sp(8.0) + sp(8.0))) < 1e-12
    # the same two negatives both as subjects: <E2,E1>=8 and <E3,E1>=16
    assert abs(orc.loss_kge(E, R, d, [0], [0], [1], [2, 3], 2, 0) - (sp(-2.0) + sp(8.0) + sp(16.0))) < 1e-12


def test_adagrad_closed_form_accumulation_and_nonlinearity():
    d = 2
    uniq = np.array([1], np.uint32)
    C = __import__("ctypes")
    def apply(T, G, delta, lr=0.5, eps=1e-10):
        acc = np.array(delta, np.float64)
        orc.lib().nor_apply_adagrad_rows(T.ctypes.data_as(C.POINTER(C.c_float)), G.ctypes.data_as(C.POINTER(C.c_float)),
                                         C.c_int32(64), C.c_int32(d), uniq.ctypes.data_as(C.POINTER(C.c_uint32)),
                                         C.c_int64(1), acc.ctypes.data_as(C.POINTER(C.c_double)),
                                         C.c_float(lr), C.c_float(eps))
    T = np.zeros((2, 64), np.float32); G = np.zeros_like(T)
    apply(T, G, [3.0, -4.0])
    assert np.allclose(G[1, :2], [9, 16]) and np.allclose(T[1, :2], [-0.5, 0.5])       # theta - lr * sign
    apply(T, G, [4.0, 3.0])
    assert np.allclose(G[1, :2], [25, 25])                                             # state accumulates
    assert np.allclose(T[1, :2], [-0.5 - 0.5 * 4 / 5, 0.5 - 0.5 * 3 / 5])
    assert np.all(T[0] == 0) and np.all(G[0] == 0)
    # two updates with g differ from one update with 2g: aggregation has to come before the update
    T2 = np.zeros((2, 64), np.float32); G2 = np.zeros_like(T2)
    apply(T2, G2, [2.0, 2.0]); apply(T2, G2, [2.0, 2.0])
    T3 = np.zeros((2, 64), np.float32); G3 = np.zeros_like(T3)
    apply(T3, G3, [4.0, 4.0])
    assert abs(T2[1, 0] - (-0.5 - 0.5 * 2 / np.sqrt(8))) < 1e-6 and abs(T3[1, 0] + 0.5) < 1e-6


def test_kge_duplicate_entities_are_aggregated_before_adagrad():
    # same triple twice in a batch: summed gradient 2g, so G = (2g)^2, not 2 g^2
    rng = np.random.default_rng(5)
    d = 4
    E, R = _rows(rng, 3, d), _rows(rng, 1, d)
    one = [E.copy(), np.zeros_like(E), R.copy(), np.zeros_like(R)]
    two = [E.copy(), np.zeros_like(E), R.copy(), np.zeros_like(R)]
    orc.step_kge(*one, d, [0], [0], [1], [2], 1, 0, 0.1, 1e-10)
    orc.step_kge(*two, d, [0, 0], [0, 0], [1, 1], [2, 2], 1, 0, 0.1, 1e-10)
    assert np.allclose(two[1], 4 * one[1], rtol=1e-6) and np.allclose(two[3], 4 * one[3], rtol=1e-6)


# ----------------------------------------------------------------------------- pull / push
def test_pull_returns_one_copy_per_position_and_push_sums_duplicates():
    rng = np.random.default_rng(0)
    T = _quantised(rng, (5, 3), 64)
    got = orc.pull(T, [4, 0, 4])
    assert np.array_equal(got[0], T[4]) and np.array_equal(got[1], T[0]) and np.array_equal(got[2], T[4])
    upd = np.zeros((3, 64), np.float32); upd[:, :3] = [[1, 2, 3], [10, 20, 30], [0.5, 0.25, 0.125]]
    T1 = T.copy(); orc.push(T1, 3, [4, 0, 4], upd)
    T2 = T.copy(); summed = np.zeros((2, 64), np.float32); summed[0] = upd[0] + upd[2]; summed[1] = upd[1]
    orc.push(T2, 3, [4, 0], summed)
    assert np.array_equal(T1, T2)
    assert np.array_equal(T1[4, :3], T[4, :3] + np.float32([1.5, 2.25, 3.125]))
    assert np.array_equal(T1[1:4], T[1:4])
    with pytest.raises(ValueError):
        orc.pull(T, [5])
