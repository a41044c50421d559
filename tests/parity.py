"""Shared helpers of the GPU parity tests."""
import numpy as np


def max_rel_err(got: np.ndarray, ref: np.ndarray, cols=None):
    """max_i |got_i - ref_i| / max(|ref_i|, tau) with tau = 1e-3 * RMS(ref), over the logical lanes `cols`.
    Also returns the maximum absolute error."""
    if cols is not None:
        got, ref = got[:, cols], ref[:, cols]
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    tau = 1e-3 * np.sqrt(np.mean(ref * ref))
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
