"""ctypes binding of libnups.so: the same entry points as include/nups.h, argument marshalling only.

Device arrays are passed as torch tensors (or raw integer addresses); PyTorch supplies the
device memory and the stream, every computation happens inside the library's kernels.
Opening the library fails loudly if it has not been built; there is no fallback path.
"""

from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnups.so")

NUPS_OK, NUPS_ERR_ARG, NUPS_ERR_KEY_RANGE, NUPS_ERR_OVERPULL = 0, -1, -2, -3
NUPS_ERR_STATE, NUPS_ERR_DEVICE, NUPS_ERR_UNIMPLEMENTED = -4, -5, -6
NUPS_CONFORM, NUPS_BOUNDED, NUPS_LONGTERM, NUPS_NONCONFORM = 1, 2, 3, 4
NUPS_TASK_SGNS, NUPS_TASK_MF, NUPS_TASK_KGE = 1, 2, 3
NUPS_STATIC_MAX_PUSH, NUPS_STATIC_MAX_KEYS = 16384, 1048576
(NUPS_PHASE_SAMPLE, NUPS_PHASE_PLAN, NUPS_PHASE_GRAD, NUPS_PHASE_APPLY0, NUPS_PHASE_APPLY1, NUPS_PHASE_PULL,
 NUPS_PHASE_PUSH, NUPS_PHASE_COUNT) = range(8)

EXPORTS = [
    "nups_init", "nups_destroy", "nups_set_state", "nups_set_hot_keys", "nups_set_deterministic",
    "nups_set_replicas", "nups_sync_replicas", "nups_replica_rows",
    "nups_set_update_clipping",
    "nups_get_update_clipping", "nups_pull", "nups_push", "nups_push_static",
    "nups_build_alias_table", "nups_register_distribution", "nups_register_distribution_at_level",
    "nups_select_hot_keys", "nups_set_local_keys", "nups_set_postponing", "nups_prepare_sample",
    "nups_pull_sample", "nups_sample_keys", "nups_release_sample", "nups_step", "nups_prepare_step",
    "nups_step_prepared", "nups_debug_structure",
    "nups_check", "nups_profile", "nups_profile_read", "nups_phase_name", "nups_last_error",
]


class NupsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("nups status %d: %s" % (status, message))
        self.status = status


class nups_batch(C.Structure):
    _fields_ = [("task", C.c_int32), ("B", C.c_int64), ("k0", C.c_void_p), ("k1", C.c_void_p), ("k2", C.c_void_p),
                ("val", C.c_void_p), ("n_neg", C.c_int32), ("n_neg2", C.c_int32), ("lr", C.c_float),
                ("l2", C.c_float), ("eps", C.c_float), ("negs", C.c_void_p), ("sample", C.c_void_p),
                ("dist", C.c_void_p), ("sample_step", C.c_uint64)]


_lib = None


def lib():
    """Opens libnups.so (built by build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(LIB_PATH + " is missing: run `python -m paper_2104_00501_amd.build` "
                                    "(or __graft_entry__.build()) first")
        _lib = C.CDLL(LIB_PATH)
        _lib.nups_last_error.restype = C.c_char_p
        _lib.nups_phase_name.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("nups_last_error", "nups_phase_name"):
                getattr(_lib, name).restype = C.c_int
    return _lib


def _check(status):
    if status != NUPS_OK:
        raise NupsError(status, (lib().nups_last_error() or b"").decode())


def _ptr(x):
    """Device (or host) address of a tensor / numpy array / int / None."""
    if x is None:
        return C.c_void_p(None)
    if isinstance(x, int):
        return C.c_void_p(x)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    return C.c_void_p(x.ctypes.data)


def nups_last_error() -> str:
    return (lib().nups_last_error() or b"").decode()


def nups_phase_name(phase: int) -> str:
    return (lib().nups_phase_name(C.c_int(phase)) or b"").decode()


def nups_init(tables, dims, stream=None):
    """tables: list of [num_keys, row_stride] fp32 device tensors; dims: logical row lengths.
    stream: a torch.cuda.Stream, a raw hipStream_t integer, or None for torch's current stream."""
    import torch
    n = len(tables)
    for t in tables:
        if t.dtype != torch.float32 or t.dim() != 2 or not t.is_contiguous():
            raise TypeError("tables must be contiguous 2-D float32 tensors")
    ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in tables])
    nk = (C.c_int64 * n)(*[t.shape[0] for t in tables])
    dm = (C.c_int32 * n)(*[int(d) for d in dims])
    rs = (C.c_int32 * n)(*[t.shape[1] for t in tables])
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    ctx = C.c_void_p(None)
    _check(lib().nups_init(C.byref(ctx), C.c_int(n), ptrs, nk, dm, rs, C.c_void_p(stream)))
    return ctx


def nups_destroy(ctx):
    _check(lib().nups_destroy(ctx))


def nups_set_state(ctx, table, state):
    _check(lib().nups_set_state(ctx, C.c_int(table), _ptr(state)))


def nups_set_hot_keys(ctx, table, keys_host):
    import numpy as np
    k = np.ascontiguousarray(keys_host, dtype=np.uint32)
    _check(lib().nups_set_hot_keys(ctx, C.c_int(table), _ptr(k) if len(k) else C.c_void_p(None), C.c_int64(len(k))))


def nups_set_replicas(ctx, replicas):
    _check(lib().nups_set_replicas(ctx, C.c_int32(replicas)))


def nups_sync_replicas(ctx):
    _check(lib().nups_sync_replicas(ctx))


def nups_replica_rows(ctx, table):
    """Returns (device address, number of rows) of the table's replica buffer."""
    rows, n = C.c_void_p(None), C.c_int64(0)
    _check(lib().nups_replica_rows(ctx, C.c_int(table), C.byref(rows), C.byref(n)))
    return rows.value, n.value


def nups_set_deterministic(ctx, enable):
    _check(lib().nups_set_deterministic(ctx, C.c_int(1 if enable else 0)))


def nups_set_update_clipping(ctx, factor):
    _check(lib().nups_set_update_clipping(ctx, C.c_float(factor)))


def nups_get_update_clipping(ctx, table):
    """Returns (sum of the recorded norms, their number)."""
    norm_sum, norm_count = C.c_double(0.0), C.c_double(0.0)
    _check(lib().nups_get_update_clipping(ctx, C.c_int(table), C.byref(norm_sum), C.byref(norm_count)))
    return norm_sum.value, norm_count.value


def nups_pull(ctx, table, keys, n, values):
    _check(lib().nups_pull(ctx, C.c_int(table), _ptr(keys), C.c_int64(n), _ptr(values)))


def nups_push_static(ctx, table, keys, n, updates):
    _check(lib().nups_push_static(ctx, C.c_int(table), _ptr(keys), C.c_int64(n), _ptr(updates)))


def nups_push(ctx, table, keys, n, updates):
    _check(lib().nups_push(ctx, C.c_int(table), _ptr(keys), C.c_int64(n), _ptr(updates)))


def nups_build_alias_table(weights_host):
    """Host only.  Returns (thresh, alias) uint32 numpy arrays."""
    import numpy as np
    w = np.ascontiguousarray(weights_host, dtype=np.float64)
    thresh = np.zeros(len(w), dtype=np.uint32)
    alias = np.zeros(len(w), dtype=np.uint32)
    _check(lib().nups_build_alias_table(_ptr(w), C.c_int64(len(w)), _ptr(thresh), _ptr(alias)))
    return thresh, alias


def nups_register_distribution(ctx, table, weights_host, scheme, U=1, G=1, P=1, R=1, seed=0):
    import numpy as np
    w = None if weights_host is None else np.ascontiguousarray(weights_host, dtype=np.float64)
    dist = C.c_void_p(None)
    _check(lib().nups_register_distribution(ctx, C.c_int(table), _ptr(w), C.c_int(scheme), C.c_int32(U),
                                            C.c_int32(G), C.c_int64(P), C.c_int32(R), C.c_uint64(seed),
                                            C.byref(dist)))
    return dist


def nups_register_distribution_at_level(ctx, table, weights_host, level, seed=0):
    import numpy as np
    w = None if weights_host is None else np.ascontiguousarray(weights_host, dtype=np.float64)
    dist = C.c_void_p(None)
    _check(lib().nups_register_distribution_at_level(ctx, C.c_int(table), _ptr(w), C.c_int(level), C.c_uint64(seed),
                                                     C.byref(dist)))
    return dist


def nups_select_hot_keys(frequency_host, factor=100.0):
    """Host only.  Returns the hot keys, most frequent first, as a uint32 numpy array."""
    import numpy as np
    f = np.ascontiguousarray(frequency_host, dtype=np.float64)
    k = C.c_int64(0)
    _check(lib().nups_select_hot_keys(_ptr(f), C.c_int64(len(f)), C.c_double(factor), C.c_void_p(None), C.c_int64(0),
                                      C.byref(k)))
    keys = np.zeros(max(k.value, 1), dtype=np.uint32)
    _check(lib().nups_select_hot_keys(_ptr(f), C.c_int64(len(f)), C.c_double(factor), _ptr(keys), C.c_int64(k.value),
                                      C.byref(k)))
    return keys[:k.value]


def nups_set_local_keys(dist, keys_a, keys_b, n_examples, per_example, split, tile):
    _check(lib().nups_set_local_keys(dist, _ptr(keys_a), _ptr(keys_b), C.c_int64(n_examples),
                                     C.c_int32(per_example), C.c_int32(split), C.c_int32(tile)))


def nups_set_postponing(dist, enable):
    _check(lib().nups_set_postponing(dist, C.c_int(1 if enable else 0)))


def nups_prepare_sample(dist, n, step):
    handle = C.c_void_p(None)
    _check(lib().nups_prepare_sample(dist, C.c_int64(n), C.c_uint64(step), C.byref(handle)))
    return handle


def nups_pull_sample(handle, n_j, keys, values=None):
    _check(lib().nups_pull_sample(handle, C.c_int64(n_j), _ptr(keys), _ptr(values)))


def nups_sample_keys(handle):
    """Returns (device address of the keys, N)."""
    p = C.c_void_p(None)
    n = C.c_int64(0)
    _check(lib().nups_sample_keys(handle, C.byref(p), C.byref(n)))
    return p.value, n.value


def nups_release_sample(handle):
    _check(lib().nups_release_sample(handle))


def make_batch(task, B, k0, k1, k2=None, val=None, n_neg=0, n_neg2=0, lr=0.0, l2=0.0, eps=0.0, negs=None, sample=None,
               dist=None, sample_step=0):
    b = nups_batch()
    b.task, b.B = task, B
    b.k0, b.k1, b.k2, b.val, b.negs = (_ptr(x).value for x in (k0, k1, k2, val, negs))
    b.n_neg, b.n_neg2, b.lr, b.l2, b.eps = n_neg, n_neg2, lr, l2, eps
    b.sample = sample.value if hasattr(sample, "value") else sample
    b.dist = dist.value if hasattr(dist, "value") else dist
    b.sample_step = sample_step
    return b


def nups_step(ctx, batch, want_loss=False):
    """Enqueues one step; with want_loss waits and returns the batch loss."""
    if want_loss:
        loss = C.c_double(0.0)
        _check(lib().nups_step(ctx, C.byref(batch), C.byref(loss)))
        return loss.value
    _check(lib().nups_step(ctx, C.byref(batch), None))
    return None


def nups_prepare_step(ctx, batch):
    """Hands a step to the library ahead of time: its key-only preparatory work then rides in the launches of the
    steps that run before it; returns the prepared step."""
    p = C.c_void_p(None)
    _check(lib().nups_prepare_step(ctx, C.byref(batch), C.byref(p)))
    return p


def nups_step_prepared(ctx, prepared, want_loss=False):
    if want_loss:
        loss = C.c_double(0.0)
        _check(lib().nups_step_prepared(ctx, prepared, C.byref(loss)))
        return loss.value
    _check(lib().nups_step_prepared(ctx, prepared, None))
    return None


def nups_debug_structure(ctx, table, uniq_keys, counts):
    n = C.c_int64(0)
    _check(lib().nups_debug_structure(ctx, C.c_int(table), _ptr(uniq_keys), _ptr(counts), C.byref(n)))
    return n.value


def nups_check(ctx):
    _check(lib().nups_check(ctx))


def nups_profile(ctx, enable):
    _check(lib().nups_profile(ctx, C.c_int(1 if enable else 0)))


def nups_profile_read(ctx, phase):
    """Returns (milliseconds, bracket count) accumulated for a phase and resets them."""
    ms = C.c_double(0.0)
    n = C.c_int64(0)
    _check(lib().nups_profile_read(ctx, C.c_int(phase), C.byref(ms), C.byref(n)))
    return ms.value, n.value
