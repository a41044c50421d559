"""Shared helpers of the GPU parity tests: the error metrics and their bars.

Two element-wise checks of a table against the oracle's, both with a floor PER ROW (never per table: with
skewed keys a table-wide scale is set by the hot rows and would hide errors in the cold ones):

* parameter error   |got_i - ref_i| / max(|ref_i|, |before_i|, tau_r)
  tau_r = RMS over the logical lanes of row r of max(|ref|, |before|).  `before` is the table as it was before the
  steps.  The element's own magnitudes come first; the row floor is there for elements that end near zero by
  cancellation: an fp32 result cannot be more accurate than about 6e-8 of what was added up to make it, and what is
  added up at lane i of a row is of the size of the row's other lanes.
* update error      max(0, |dgot_i - dref_i| - ulp_i) / max(|dref_i|, tauD_r),   d = table - before,
  tauD_r = RMS over the row's logical lanes of dref, ulp_i = 2^-23 max(|ref_i|, |before_i|): the stored fp32
  parameter quantises the applied update by up to one unit in its last place, whatever the gradient's accuracy;
  beyond that the update (learning rate x summed gradient) must itself be right to the bar.  This is the check
  that sees a wrong gradient behind a large parameter.  Where contributions to one element cancel (a negative
  that equals the context word: coefficients near +1/2 and -1/2 on the same source row), the net update says
  nothing about the size of what was added up; a test may then pass `gross`, an element-wise bound on
  learning rate x sum of |source rows| (coefficients bounded by one), as a further floor.

Rows that the oracle leaves untouched must be bit-identical to `before`.
"""
import numpy as np

TOL_ONE_STEP = 1e-5       # parameters after one step
TOL_100_STEPS = 1e-3      # parameters after 100 steps
TOL_UPDATE = 2e-5         # the applied update of one step (fp32 sums of up to thousands of products)


def _rows_rms(x):
    return np.sqrt(np.mean(x * x, axis=1, keepdims=True))


def param_err(got: np.ndarray, ref: np.ndarray, before: np.ndarray, cols=None):
    """Returns (max parameter error with the per-row floor, max absolute error)."""
    if cols is not None:
        got, ref, before = got[:, cols], ref[:, cols], before[:, cols]
    if got.size == 0:
        return 0.0, 0.0
    got, ref, before = (x.astype(np.float64) for x in (got, ref, before))
    mag = np.maximum(np.abs(ref), np.abs(before))
    den = np.maximum(mag, np.maximum(_rows_rms(mag), 1e-30))
    diff = np.abs(got - ref)
    return float(np.max(diff / den)), float(np.max(diff))


def update_err(got: np.ndarray, ref: np.ndarray, before: np.ndarray, cols=None, gross=None):
    """Max error of the applied update (table - before) with the per-row floor, net of one ulp of the parameter."""
    if cols is not None:
        got, ref, before = got[:, cols], ref[:, cols], before[:, cols]
        gross = None if gross is None else gross[:, cols]
    if got.size == 0:
        return 0.0
    got, ref, before = (x.astype(np.float64) for x in (got, ref, before))
    dref, dgot = ref - before, got - before
    touched = np.any(dref != 0, axis=1)
    if not touched.any():
        return 0.0
    dref, dgot, mag = dref[touched], dgot[touched], np.maximum(np.abs(ref), np.abs(before))[touched]
    excess = np.maximum(np.abs(dgot - dref) - mag * 2.0 ** -23, 0.0)
    den = np.maximum(np.abs(dref), np.maximum(_rows_rms(dref), 1e-30))
    if gross is not None:
        den = np.maximum(den, gross[touched])
    return float(np.max(excess / den))


def sgns_gross_updates(In, Out, center, context, negs, K, lr):
    """Element-wise bound on what one SGNS step adds up per row: lr x sum of |source row| over the row's
    accesses (every coefficient sigma(z) - label is below one in magnitude).  Only a scale for update_err."""
    B = len(center)
    okeys = np.concatenate([np.asarray(context).reshape(B, 1), np.asarray(negs).reshape(B, K)], axis=1)
    g_in, g_out = np.zeros(In.shape), np.zeros(Out.shape)
    np.add.at(g_in, np.repeat(center, K + 1), np.abs(Out[okeys.ravel()]))
    np.add.at(g_out, okeys.ravel(), np.abs(In[np.repeat(center, K + 1)]))
    return lr * g_in, lr * g_out


def untouched_rows_identical(got: np.ndarray, ref: np.ndarray, before: np.ndarray) -> bool:
    """Rows that the oracle did not change are bit-identical to their initial value in `got`."""
    same = np.all(ref == before, axis=1)
    return bool(np.array_equal(got[same], before[same]))


def assert_table(got, ref, before, cols, tol, what, tol_update=TOL_UPDATE, gross=None):
    """Both checks, the untouched rows and the padding lanes; prints the measured figures."""
    rel, ab = param_err(got, ref, before, cols)
    ue = update_err(got, ref, before, cols, gross)
    print("%s: parameter err %.3g (abs %.3g), update err %.3g" % (what, rel, ab, ue))
    assert rel <= tol, "%s: parameter error %.3g (abs %.3g) > %.1g" % (what, rel, ab, tol)
    if tol_update is not None:
        assert ue <= tol_update, "%s: update error %.3g > %.1g" % (what, ue, tol_update)
    assert untouched_rows_identical(got, ref, before), what + ": a row that the step does not touch changed"
    pad = np.setdiff1d(np.arange(got.shape[1]), cols)
    assert np.all(got[:, pad] == 0), what + ": padding lanes changed"


def dev(x, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def dev_u32(x):
    """uint32 keys as an int32-typed device tensor with the same bits."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint32).view(np.int32)).cuda()


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)
