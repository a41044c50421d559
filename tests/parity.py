"""Shared helpers of the GPU parity tests."""
import numpy as np


def max_rel_err(got: np.ndarray, ref: np.ndarray, cols=None):
    """max_i |got_i - ref_i| / max(|ref_i|, tau) with tau = RMS(ref), over the logical lanes `cols`.

    The floor tau is the scale of the stored operands: an fp32 parameter of magnitude m cannot be
    updated more accurately than about 6e-8 * m, so an element that ends near zero by cancellation
    is judged against the magnitude of what was added up, not against its own value.
    Also returns the maximum absolute error."""
    if cols is not None:
        got, ref = got[:, cols], ref[:, cols]
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    tau = np.sqrt(np.mean(ref * ref))
    diff = np.abs(got - ref)
    if diff.size == 0:
        return 0.0, 0.0
    return float(np.max(diff / np.maximum(np.abs(ref), max(tau, 1e-30)))), float(np.max(diff))


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


def update_err(got: np.ndarray, ref: np.ndarray, before: np.ndarray, cols=None):
    """Error of the applied update (table - before) relative to the RMS update of the touched rows."""
    if cols is not None:
        got, ref, before = got[:, cols], ref[:, cols], before[:, cols]
    dref = ref.astype(np.float64) - before
    dgot = got.astype(np.float64) - before
    touched = np.any(dref != 0, axis=1)
    if not touched.any():
        return 0.0
    scale = np.sqrt(np.mean(dref[touched] ** 2))
    return float(np.max(np.abs(dgot - dref)) / max(scale, 1e-30))
