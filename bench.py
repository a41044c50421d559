#!/usr/bin/env python3
"""Throughput of the sparse-SGD minibatch step on one MI355X.

Workload (default): the large skip-gram configuration -- 1M keys, d = 300 (rows padded to 320
floats), 3 negatives per pair from unigram^0.75 under BOUNDED sample reuse (U = 4, pools of 250),
batches of 16,384 (center, context) pairs cut in stream order from an i.i.d. Zipf(1.0) token
stream with window 5, learning rate 0.025 linearly decayed.  One step = draw negatives, build the
per-key aggregation structure, score + gradient, aggregate and push, all inside the timed region;
inputs (pair arrays, tables, alias table) are resident in HBM before timing starts.

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

WORKLOADS = {
    # name: V, d, K, scheme, U, G, B, window, zipf s, lr0, tokens in the full stream
    "sgns_1m_d300_bounded_u4": dict(V=1_000_000, d=300, K=3, U=4, G=250, B=16_384, window=5, s=1.0, lr0=0.025,
                                    stream_tokens=1_000_000_000, seed=1004),
    "sgns_10k_d100_conform": dict(V=10_000, d=100, K=5, U=1, G=1, B=4096, window=2, s=1.0, lr0=0.025,
                                  stream_tokens=1_000_000, seed=1001),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="sgns_1m_d300_bounded_u4", choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps to time (-1: about 15 s worth, 0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch

    from paper_2104_00501_amd import binding as nb
    from paper_2104_00501_amd import workloads as wl

    cfg = WORKLOADS[args.workload]
    V, d, K, U, G, B, window = cfg["V"], cfg["d"], cfg["K"], cfg["U"], cfg["G"], cfg["B"], cfg["window"]
    total_steps = args.warmup + args.steps
    epoch_steps = max(1, wl.num_window_pairs(cfg["stream_tokens"], window) // B)
    torch.cuda.set_device(0)

    # ---- inputs, generated once and made resident --------------------------------------------
    n_tokens = min(cfg["stream_tokens"], total_steps * B // (2 * window) + 2 * window + 2)
    toks = wl.zipf_stream(V, cfg["s"], n_tokens, cfg["seed"])
    centers, contexts = wl.window_pairs(toks, window, 0, total_steps * B)
    total_steps = len(centers) // B
    steps = total_steps - args.warmup
    assert steps > 0, "not enough pairs for the requested steps"
    weights = wl.expected_unigram_weights(V, cfg["s"], cfg["stream_tokens"])
    In, Out = wl.sgns_tables(V, d, cfg["seed"])
    stride = In.shape[1]

    def keys(x):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint32).view(np.int32)).cuda()

    tin, tout = torch.from_numpy(In).cuda(), torch.from_numpy(Out).cuda()
    kc, ko = keys(centers), keys(contexts)
    ctx = nb.nups_init([tin, tout], [d, d])
    scheme = nb.NUPS_BOUNDED if U > 1 else nb.NUPS_CONFORM
    dist = nb.nups_register_distribution(ctx, 1, weights, scheme, U=U, G=G, seed=cfg["seed"])
    lrs = [float(wl.linear_lr(cfg["lr0"], t, epoch_steps)) for t in range(total_steps)]

    def prepare(t):
        """The key-only half of step t on the library's side stream: draw the negatives, build the plan."""
        batch = nb.make_batch(nb.NUPS_TASK_SGNS, B, kc.data_ptr() + 4 * t * B, ko.data_ptr() + 4 * t * B,
                              n_neg=K, lr=lrs[t], dist=dist, sample_step=t)
        return nb.nups_prepare_step(ctx, batch)

    def run(first, count):
        # software pipeline: step t+1 is prepared before step t runs, so the two overlap on the GPU
        nxt = prepare(first)
        for t in range(first, first + count):
            p = nxt
            if t + 1 < first + count:
                nxt = prepare(t + 1)
            nb.nups_step_prepared(ctx, p)

    # ---- warm-up, then the timed region ---------------------------------------------------------
    run(0, args.warmup)
    nb.nups_check(ctx)
    snap_in, snap_out = tin.clone(), tout.clone()       # state after warm-up, for the profiling pass
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.warmup, steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    nb.nups_check(ctx)
    ms_per_step = 1e3 * elapsed / steps
    value = steps * B / elapsed

    # ---- per-kernel pass: same steps, HIP events around every phase on the library's stream -----
    tin.copy_(snap_in)
    tout.copy_(snap_out)
    torch.cuda.synchronize()
    nb.nups_profile(ctx, True)
    uk = torch.zeros(B * (K + 1), dtype=torch.int32, device="cuda")
    uc = torch.zeros(B * (K + 1), dtype=torch.int32, device="cuda")
    n_struct = min(steps, 32)
    nu_in = nu_out = 0
    for t in range(args.warmup, args.warmup + steps):
        run(t, 1)
        if t - args.warmup < n_struct:                   # distinct rows per step, for the algorithmic bytes
            nu_in += nb.nups_debug_structure(ctx, 0, uk, uc)
            nu_out += nb.nups_debug_structure(ctx, 1, uk, uc)
    nu_in /= n_struct
    nu_out /= n_struct
    phases = {}
    for p in range(nb.NUPS_PHASE_COUNT):
        ms, n = nb.nups_profile_read(ctx, p)
        if n:
            phases[nb.nups_phase_name(p)] = {"ms_per_step": ms / steps, "brackets": n}
    nb.nups_profile(ctx, False)

    # a plain copy of known size through the library's own gather kernel (rows 0..n-1 in order): the
    # reference that hardware byte counters are scaled with
    n_cal = min(V, 262_144)
    cal_keys = torch.arange(n_cal, dtype=torch.int32, device="cuda")
    cal_out = torch.empty((n_cal, stride), dtype=torch.float32, device="cuda")
    nb.nups_pull(ctx, 0, cal_keys, n_cal, cal_out)
    torch.cuda.synchronize()
    del cal_out

    # Algorithmic bytes per step under snapshot semantics: every distinct touched row is read once
    # and written once (4 * d bytes each way), plus the key arrays (4 bytes per access).
    row_bytes = 4 * d
    alg = {
        "grad": (nu_in + nu_out) * row_bytes + 4 * B * (2 + K) + 4 * B * (K + 1),   # read rows, keys; write coefficients
        "apply0": nu_in * row_bytes * 2 + 4 * B,                                      # input table read-modify-write
        "apply1": nu_out * row_bytes * 2 + 4 * B * (K + 1) * 2,                       # output table rmw, keys + coefficients
    }
    step_alg_bytes = (nu_in + nu_out) * row_bytes * 2 + 4 * B * (2 + K)
    dominant = max((p for p in alg if p in phases), key=lambda p: phases[p]["ms_per_step"])
    dom_ms = phases[dominant]["ms_per_step"]
    achieved = alg[dominant] / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                "algorithmic_bytes_per_launch": alg[dominant], "kernel_ms": dom_ms,
                "whole_step_algorithmic_GBps": step_alg_bytes / (ms_per_step * 1e-3) / 1e9,
                "whole_step_logical_GBps": B * (2 + K) * row_bytes * 3 / (ms_per_step * 1e-3) / 1e9,
                "distinct_rows_per_step": {"input": nu_in, "output": nu_out}}

    # ---- CPU baseline: the oracle, as it stands, on a prefix of the same steps -------------------
    cpu = None
    if args.cpu_steps != 0:
        from oracle import oracle as orc
        alias = orc.alias_build(weights)
        oin, oout = In, Out                              # host tables (fresh initial values)
        n_cpu = args.cpu_steps if args.cpu_steps > 0 else 10 ** 9
        done, t_cpu = 0, time.perf_counter()
        while done < min(n_cpu, total_steps):
            c, o = centers[done * B:(done + 1) * B], contexts[done * B:(done + 1) * B]
            if U > 1:
                ng = orc.sample_bounded(alias, V, cfg["seed"], 0, done, B * K, U, G)
            else:
                ng = orc.sample_conform(alias, V, cfg["seed"], 0, done, B * K)
            orc.step_sgns(oin, oout, d, c, o, ng, K, lrs[done])
            done += 1
            if args.cpu_steps < 0 and time.perf_counter() - t_cpu > 15.0:
                break
        dt = time.perf_counter() - t_cpu
        cpu = {"value": done * B / dt, "unit": "positive examples/s", "cores": 1, "kind": "oracle",
               "sample": "first %d steps of the same workload (%d pairs), single thread, %.1f s" % (done, done * B, dt),
               "host_cores_available": os.cpu_count()}

    out = {
        "metric": "positive examples/sec per step (pull+grad+push)", "value": value, "unit": "positive examples/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "num_keys": V, "dim": d, "row_stride": stride, "negatives": K,
                   "scheme": "BOUNDED U=%d G=%d" % (U, G) if U > 1 else "CONFORM", "batch": B, "window": window,
                   "zipf_s": cfg["s"], "lr0": cfg["lr0"], "pairs": "stream order"},
        "roofline": roofline, "phases_ms_per_step": {k: v["ms_per_step"] for k, v in phases.items()},
        "cpu_baseline": cpu,
        "finite": bool(torch.isfinite(tin).all().item() and torch.isfinite(tout).all().item()),
    }
    nb.nups_destroy(ctx)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
