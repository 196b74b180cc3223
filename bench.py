#!/usr/bin/env python3
"""Benchmark of the Zeno aggregation step on one MI355X.

One step = one whole aggregation: zeno_score over the m candidates followed by
zeno_aggregate (selection + average), on seeded synthetic inputs that are
already resident in HBM.  Prints ONE JSON line: aggregations/s, the roofline
figures of the dominant kernel (the candidate layer kernel that streams G),
measured with HIP events around every launch, and the CPU oracle timed on a
bounded sample of the same workload as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the largest, 14 GB of candidates)")
    ap.add_argument("--buffers", type=int, default=0,
                    help="distinct copies of G to rotate over (0 = automatic: enough to defeat the 256 MB cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain elementwise copy-like kernel (torch.ceil, 4 GiB in, 4 GiB out) so that rocprofv3 "
                         "byte counters collected over this command can be scaled")
    ap.add_argument("--row-align", type=int, default=32,
                    help="alignment of the rows of G in floats (32 = 128-byte lines, the layout the library "
                         "recommends; 1 = densely packed rows)")
    ap.add_argument("--n-r", type=int, default=0,
                    help="override the size of the server's batch (0 = the workload's own; the paper's runs use 4)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the CPU oracle sample")
    return ap.parse_args()


def cpu_baseline(w, budget_s):
    """The float64 oracle, as it stands, on a bounded sample: f_r(x) once, k of the
    m candidates, and the selection + average on the first d_s coordinates; the
    parts are scaled to the full step."""
    import numpy as np
    import torch
    from oracle import zeno_oracle as O

    npy = lambda t: None if t is None else t.detach().cpu().numpy()
    x = npy(w.x)
    feats, labels, targets = npy(w.features), npy(w.labels), npy(w.targets)
    args = (w.dims, w.has_bias, w.loss, feats, labels, targets)
    t0 = time.perf_counter()
    f0 = O.f_r(x.astype(np.float64), *args)
    t_f0 = time.perf_counter() - t0
    k, t_cand = 0, 0.0
    while k < w.m and (k < 1 or t_cand + t_cand / max(k, 1) < budget_s * 0.7):
        u = npy(w.G[k])
        t0 = time.perf_counter()
        O.score(x, u, w.gamma, w.rho, f0, *args)
        t_cand += time.perf_counter() - t0
        k += 1
    d_s = min(w.d, max(1, int(2.0e8 // (4 * w.m))))     # ~200 MB of candidate columns
    Gs = npy(w.G[:, :d_s])
    s = np.random.default_rng(0).normal(size=w.m)
    t0 = time.perf_counter()
    O.zeno_aggregate(Gs, s, w.b)
    t_agg = (time.perf_counter() - t0) * (w.d / d_s)
    total = t_f0 + t_cand * (w.m / k) + t_agg
    return {"value": 1.0 / total, "unit": "aggregations/s", "cores": torch.get_num_threads(),
            "kind": "oracle",
            "sample": f"f_r(x) + {k} of {w.m} candidates scored + selection/average on {d_s} of {w.d} "
                      f"coordinates, scaled to the full step ({total:.2f} s)"}


def read_traffic(cfg):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3
    counter summary, if there is one for this workload."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"traffic_cfg{cfg}.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    a = parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: the Zeno step here has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1805_10032_amd import binding as B, workloads as WL

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.load_library()
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    w = WL.make_config(a.config, device=dev, row_align=a.row_align, n_r=a.n_r or None)
    m, d, b = w.m, w.d, w.b
    g_bytes = 4 * m * d
    if a.buffers > 0:
        n_buf = a.buffers
    elif g_bytes >= (1 << 30):
        n_buf = 1               # far larger than the 256 MB last-level cache
    else:
        n_buf = min(8, (1 << 30) // g_bytes + 1)
    Gs = [w.G]
    for _ in range(n_buf - 1):
        Gs.append(WL._alloc_rows(m, d, a.row_align, dev))
        Gs[-1].copy_(w.G)
    mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
    ws = B.alloc_workspace(mdl, m, w.n_r, dev)
    scores = torch.empty(m, dtype=torch.float32, device=dev)
    out = torch.empty(d, dtype=torch.float32, device=dev)
    sel = torch.empty(m - b, dtype=torch.int32, device=dev)

    def step(i):
        G = Gs[i % n_buf]
        B.zeno_score(mdl, w.x, G, w.features, w.gamma, w.rho, labels=w.labels, targets=w.targets,
                     scores=scores, workspace=ws)
        B.zeno_aggregate(G, scores, b, out=out, selected=sel)

    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.ceil(src, out=dst)   # a plain elementwise kernel: reads 4 GiB, writes 4 GiB
        torch.cuda.synchronize()
        del src, dst

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / a.steps

    # per-launch durations (HIP events on the launch stream), in a separate loop so
    # that the event records do not sit inside the timed region above
    B.profile_enable(True)
    n_prof = max(3, min(a.steps, 10))
    for i in range(n_prof):
        step(i)
    torch.cuda.synchronize()
    recs = B.profile_collect()
    B.profile_enable(False)
    per, per_layer = {}, {}
    for name, layer, ms, nbytes in recs:
        if name.startswith("layer"):
            e = per_layer.setdefault(f"{name}[{layer}]", [0, 0.0, 0.0])
            e[0] += 1
            e[1] += ms
            e[2] += nbytes
        e = per.setdefault(name, [0, 0.0, 0.0])
        e[0] += 1
        e[1] += ms
        e[2] += nbytes
    # the baseline aggregators on the same G (Section 6.1.1, Definitions 4 and 5), and the variant of
    # the aggregation that also takes the server's SGD step (Algorithm 1), in place on a copy of x
    x_step = w.x.clone()
    for i in range(-1, 3):                             # the first pass is an unrecorded warm-up
        B.profile_enable(i >= 0)
        B.zeno_mean(Gs[i % n_buf], out=out)
        B.zeno_median(Gs[i % n_buf], out=out)
        B.zeno_aggregate_update(Gs[i % n_buf], scores, b, w.gamma, x_step, x_next=x_step, want_out=False,
                                selected=sel)
        if 3 <= m <= 128 and m - b - 2 >= 1:
            B.zeno_krum(Gs[i % n_buf], b, out=out)     # Krum_b (Definition 5), the paper's main baseline
    torch.cuda.synchronize()
    for name, layer, ms, nbytes in B.profile_collect():
        e = per.setdefault(name, [0, 0.0, 0.0])
        e[0] += 1
        e[1] += ms
        e[2] += nbytes
    B.profile_enable(False)
    kernels = {k: {"launches_per_step": v[0] / (3 if k in ("mean", "median", "average_update", "krum") else n_prof), "avg_ms": v[1] / v[0],
                   "algorithmic_GBps": (v[2] / v[0]) / (v[1] / v[0]) / 1e6} for k, v in per.items()}
    layers = {k: {"avg_ms": v[1] / v[0], "algorithmic_GBps": v[2] / v[1] / 1e6} for k, v in per_layer.items()}
    dom = per["layer_cand"]
    dom_avg_ms = dom[1] / dom[0]
    dom_bytes = dom[2] / dom[0]
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9
    step_bytes = 4.0 * d * (2 * m - b + 2)

    result = {
        "metric": "Zeno aggregations/sec (m candidates scored+averaged) and achieved HBM GB/s",
        "value": a.steps / elapsed,
        "unit": "aggregations/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.fwd if w.fwd == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"config {a.config}: " + "->".join(str(v) for v in w.dims) +
                               f" {w.loss}, d={d}, m={m}, b={b}, n_r={w.n_r}, gamma={w.gamma}, rho={w.rho}",
                   "G_bytes": g_bytes, "G_row_pitch_floats": int(w.G.stride(0)), "G_buffers_rotated": n_buf},
        "step_algorithmic_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "layer_kernel (candidate layers, streams G)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(a.config),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_avg_ms},
        "kernels": kernels,
        "layers": layers,
    }
    if not a.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, a.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
