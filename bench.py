#!/usr/bin/env python3
"""Benchmark of the hot path: batched 1D TV prox, forward + backward, on one MI355X.

A step is one pass of the whole path (tv1d_prox_fwd then tv1d_prox_bwd with dL/dlam) over
the 2^20-row workload ([256,128,32,32] fp32 viewed as rows of length 32, per-channel lam
log-uniform in [1e-3, 10]); inputs are resident in HBM before the timed region starts.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E peak
FWD_BYTES_PER_ELEM = 8          # read y, write x
BWD_BYTES_PER_ELEM = 12         # read g_up and x, write grad_y


def cpu_baseline(sample_rows: int):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the
    same workload (fwd + bwd), rows/s."""
    import numpy as np

    import oracle
    import workloads

    chunk_B = 64                                   # 2^18 rows per chunk keeps memory small
    n_chunks = max(1, sample_rows // (chunk_B * 128 * 32))
    oracle.prox1d_batch(np.zeros((1, 32)), np.ones(1))         # load the library
    rows, dt = 0, 0.0
    for c in range(n_chunks):
        y, lam, g = workloads.config3(B=chunk_B, C=128, salt=c)
        y64, g64, lam64 = y.astype(np.float64), g.astype(np.float64), lam.astype(np.float64)
        t0 = time.perf_counter()
        x = oracle.prox1d_batch(y64, lam64, axis=-1, lam_div=32)
        oracle.prox1d_bwd_batch(g64, x, lam_count=128, axis=-1, lam_div=32)
        dt += time.perf_counter() - t0
        rows += y.size // 32
    return {"value": rows / dt, "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d rows x 32 drawn like the workload, in %d chunks (fwd+bwd, fp64, OpenMP "
                      "over rows), %.2f s of wall time" % (rows, n_chunks, dt)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=1 << 23)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (rows are independent; see DESIGN.md for "
              "how the path would shard); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2204_03643_amd as tv
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    y, lam, g = workloads.config3()
    B, C, H, W = y.shape
    n_rows, n_elem = B * C * H, y.size
    yt, lt, gt = (torch.from_numpy(a).to(dev) for a in (y, lam, g))
    xt, gy = torch.empty_like(yt), torch.empty_like(yt)
    gl = torch.empty_like(lt)
    rows = tv.rows_along(y.shape, -1)
    L = tv.tv_lambda(lt.data_ptr(), C, H)
    wsb = tv.tv1d_bwd_workspace_bytes(rows, L)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(evs=None):
        if evs is not None:
            evs[0].record(stream)
        tv.tv1d_prox_fwd(yt, xt, rows, L, stream)
        if evs is not None:
            evs[1].record(stream)
        tv.tv1d_prox_bwd(gt, xt, gy, gl, rows, L, ws, wsb, stream)
        if evs is not None:
            evs[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    fwd_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    bwd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))   # bwd kernel + lam reduction
    ms_per_step = wall * 1e3 / args.steps
    value = n_rows * args.steps / wall

    fwd_bytes, bwd_bytes = n_elem * FWD_BYTES_PER_ELEM, n_elem * BWD_BYTES_PER_ELEM
    fwd_gbs = fwd_bytes / (fwd_ms * 1e-3) / 1e9
    bwd_gbs = bwd_bytes / (bwd_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_tv1d_fwd_short_config3.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("traffic_bytes_per_launch")

    out = {
        "metric": "TV-prox rows/s (fwd+bwd), 2^20 rows x len 32",
        "value": value,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "config 3: 2^20 rows x 32 fp32 ([256,128,32,32] ~N(0,1), per-channel "
                               "lam log-uniform [1e-3,10]), tv1d_prox_fwd + tv1d_prox_bwd",
                   "rows": n_rows, "length": W, "lam_slots": C},
        "effective_gbs_fwd_bwd": (fwd_bytes + bwd_bytes) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9,
        "effective_frac_of_hbm_peak": (fwd_bytes + bwd_bytes) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"kernel": "tv1d_fwd_short_kernel<32>", "bound": "hbm", "achieved": fwd_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fwd_gbs / HBM_PEAK_GBS,
                     "traffic": traffic, "launch_us": fwd_ms * 1e3,
                     "algorithmic_bytes_per_launch": fwd_bytes},
        "roofline_bwd": {"kernel": "tv1d_bwd_short_kernel<32> + reduce_lambda_kernel", "bound": "hbm",
                         "achieved": bwd_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": bwd_gbs / HBM_PEAK_GBS, "launch_us": bwd_ms * 1e3,
                         "algorithmic_bytes_per_launch": bwd_bytes},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample_rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
