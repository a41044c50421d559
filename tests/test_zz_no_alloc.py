"""nups_push_static, the push for callers that cannot allocate: called through the C ABI and checked against
nups_push on the same inputs, twice in a row (the second call with a smaller input), plus its size limits."""
import numpy as np
import pytest

from paper_2104_00501_amd import binding as nb
from paper_2104_00501_amd import workloads as wl
from tests.parity import TOL_ONE_STEP, TOL_UPDATE, dev, dev_u32, host_u32, param_err, update_err

pytestmark = pytest.mark.gpu


def _structure(ctx, n):
    import torch
    uk = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda")
    uc = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda")
    nu = nb.nups_debug_structure(ctx, 0, uk, uc)
    return host_u32(uk)[:nu].copy(), host_u32(uc)[:nu].copy()


@pytest.mark.parametrize("deterministic", [False, True])
def test_push_static_matches_push_on_two_calls_in_a_row(deterministic):
    V, d = 300_000, 300
    T = wl.uniform_table(V, d, -1.0, 1.0, 3)
    t_static, t_plain = dev(T), dev(T)
    ctx_s = nb.nups_init([t_static], [d])
    ctx_p = nb.nups_init([t_plain], [d])
    nb.nups_set_deterministic(ctx_s, deterministic)
    nb.nups_set_deterministic(ctx_p, deterministic)
    prev_static = prev_plain = T
    for call, (n, s, seed) in enumerate([(16_384, 1.2, 5), (3_001, 0.7, 6)]):      # the second input is smaller
        keys = wl.zipf_stream(V, s, n, seed)
        upd = wl.uniform_table(n, d, -1e-2, 1e-2, seed + 10)
        assert np.bincount(keys).max() > (600 if call == 0 else 1)                  # chunked segments in the first call
        kd, ud = dev_u32(keys), dev(upd)
        nb.nups_push_static(ctx_s, 0, kd, n, ud)
        nb.nups_check(ctx_s)
        nb.nups_push(ctx_p, 0, kd, n, ud)
        nb.nups_check(ctx_p)
        ks, cs = _structure(ctx_s, n)
        kp, cp = _structure(ctx_p, n)
        assert np.array_equal(ks, kp) and np.array_equal(cs, cp)                    # structure: bit-exact
        got, ref = t_static.cpu().numpy(), t_plain.cpu().numpy()
        if deterministic:
            assert np.array_equal(got, ref), "call %d: tables differ in deterministic mode" % call
        cols = list(range(d))
        rel, ab = param_err(got, ref, prev_plain, cols)
        ue = update_err(got, ref, prev_plain, cols)
        print("push_static vs push, call %d: parameter err %.3g (abs %.3g), update err %.3g" % (call, rel, ab, ue))
        assert rel <= TOL_ONE_STEP and ue <= call * TOL_ONE_STEP + TOL_UPDATE   # the first call's difference stays
        untouched = np.setdiff1d(np.arange(V), ks)
        assert np.array_equal(got[untouched], prev_static[untouched]), "call %d: a row without a key changed" % call
        assert np.all(got[:, d:] == 0)
        prev_static, prev_plain = got, ref
    nb.nups_push_static(ctx_s, 0, None, 0, None)                                    # an empty push is a no-op
    nb.nups_check(ctx_s)
    assert np.array_equal(t_static.cpu().numpy(), got)
    nb.nups_destroy(ctx_s)
    nb.nups_destroy(ctx_p)


def test_push_static_rejects_sizes_beyond_its_scratch():
    d = 64
    small = dev(wl.uniform_table(1000, d, -1, 1, 1))
    ctx = nb.nups_init([small], [d])
    n = nb.NUPS_STATIC_MAX_PUSH + 1
    keys, upd = dev_u32(np.zeros(n, dtype=np.uint32)), dev(np.zeros((n, 64), dtype=np.float32))
    with pytest.raises(nb.NupsError) as e:
        nb.nups_push_static(ctx, 0, keys, n, upd)
    assert e.value.status == nb.NUPS_ERR_ARG and "NUPS_STATIC_MAX_PUSH" in str(e.value)
    nb.nups_destroy(ctx)
    import torch
    big = torch.zeros((nb.NUPS_STATIC_MAX_KEYS + 1, d), dtype=torch.float32, device="cuda")
    ctx = nb.nups_init([big], [d])
    with pytest.raises(nb.NupsError) as e:
        nb.nups_push_static(ctx, 0, keys, 1, upd)
    assert e.value.status == nb.NUPS_ERR_ARG and "NUPS_STATIC_MAX_KEYS" in str(e.value)
    nb.nups_destroy(ctx)
