#!/usr/bin/env python3
"""Benchmark of the Zeno aggregation step on one MI355X.

One step = one whole aggregation: zeno_score over the m candidates followed by
zeno_aggregate (selection + average), on seeded synthetic inputs that are
already resident in HBM.  Prints ONE JSON line: aggregations/s on the headline
workload (config 5, rows of G on 128-byte lines), the roofline figures of the
dominant kernel (the candidate layer kernel that streams G), measured with HIP
events around every launch, and the CPU oracle timed on a bounded sample of the
same workload as a baseline.  The same line carries, under "also", the same
measurement for the densely packed layout G[m x d] of the headline workload,
for workload 4, for workloads 3, 2 and 1 (buffers rotated so that G comes
from HBM, eager launches and a replayed HIP graph), and for a convolutional
model of the shape of the paper's own experiments.

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
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload (no 'also' section)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain elementwise copy-like kernel (torch.ceil, 4 GiB in, 4 GiB out) so that rocprofv3 "
                         "byte counters collected over this command can be scaled")
    ap.add_argument("--row-align", type=int, default=32,
                    help="alignment of the rows of G in floats (32 = 128-byte lines, an odd number of them per row: "
                         "the layout the library recommends; 1 = densely packed rows, ld = d)")
    ap.add_argument("--n-r", type=int, default=0,
                    help="override the size of the server's batch (0 = the workload's own; the paper's runs use 4)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the CPU oracle sample")
    return ap.parse_args()


def blas_threads():
    """Threads of the BLAS library NumPy's matrix products run on (what the oracle really uses)."""
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return int(max(n))
    except Exception:
        pass
    return int(os.environ.get("OMP_NUM_THREADS", 0)) or os.cpu_count()


def cpu_baseline(w, budget_s):
    """The float64 oracle, as it stands, on a bounded sample: f_r(x) once, k of the
    m candidates, and the selection + average on the first d_s coordinates; the
    parts are scaled to the full step."""
    import numpy as np
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
    return {"value": 1.0 / total, "unit": "aggregations/s", "cores": blas_threads(), "host_cpus": os.cpu_count(),
            "kind": "oracle",
            "sample": f"f_r(x) + {k} of {w.m} candidates scored + selection/average on {d_s} of {w.d} "
                      f"coordinates, scaled to the full step ({total:.2f} s); NumPy float64, matrix products on "
                      f"{blas_threads()} BLAS threads, the rest single-threaded"}


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


class Runner:
    """One workload resident on the GPU: buffers, the step, timing and per-launch records."""

    def __init__(self, B, WL, torch, cfg, row_align, n_r=None, buffers=0, w=None):
        self.B, self.torch, self.cfg = B, torch, cfg
        dev = torch.device("cuda", 0)
        if w is None:
            w = WL.make_config(cfg, device=dev, row_align=row_align, n_r=n_r)
        elif row_align <= 1 and w.G.stride(0) != w.d:
            w = _with_G(w, w.G.contiguous())           # same values, densely packed: G[m x d], ld = d
        self.w = w
        m, d, b = w.m, w.d, w.b
        g_bytes = 4 * m * d
        if buffers > 0:
            n_buf = buffers
        elif g_bytes >= (1 << 30):
            n_buf = 1               # far larger than the 256 MB last-level cache
        else:
            n_buf = min(8, (1 << 30) // g_bytes + 1)
        self.Gs = [w.G]
        for _ in range(n_buf - 1):
            g = WL._alloc_rows(m, d, row_align, dev) if row_align > 1 else torch.empty((m, d), device=dev)
            g.copy_(w.G)
            self.Gs.append(g)
        self.n_buf = n_buf
        self.mdl = B.ZenoModel(w.dims, w.has_bias, w.loss, w.fwd)
        self.ws = B.alloc_workspace(self.mdl, m, w.n_r, dev)
        self.scores = torch.empty(m, dtype=torch.float32, device=dev)
        self.out = torch.empty(d, dtype=torch.float32, device=dev)
        self.sel = torch.empty(m - b, dtype=torch.int32, device=dev)
        self.step_bytes = 4.0 * d * (2 * m - b + 2)

    def step(self, i):
        w, B = self.w, self.B
        G = self.Gs[i % self.n_buf]
        B.zeno_score(self.mdl, w.x, G, w.features, w.gamma, w.rho, labels=w.labels, targets=w.targets,
                     scores=self.scores, workspace=self.ws)
        B.zeno_aggregate(G, self.scores, w.b, out=self.out, selected=self.sel)

    def time_steps(self, steps, warmup):
        torch = self.torch
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(i)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def time_graph(self, steps, warmup):
        """The same steps as ONE replayed HIP graph per buffer (the calls allocate nothing and never
        synchronise, so they can be captured after one eager warm-up call)."""
        torch = self.torch
        self.step(0)
        torch.cuda.synchronize()
        graphs = []
        side = torch.cuda.Stream()
        for k in range(self.n_buf):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    self.step(k)
            graphs.append(g)
        torch.cuda.synchronize()
        for i in range(warmup):
            graphs[i % self.n_buf].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i % self.n_buf].replay()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def launches(self, n_prof):
        """Per-launch durations (HIP events on the launch stream), outside the timed region."""
        B, torch = self.B, self.torch
        B.profile_enable(True)
        for i in range(n_prof):
            self.step(i)
        torch.cuda.synchronize()
        recs = B.profile_collect(detail=True)
        B.profile_enable(False)
        per, per_layer = {}, {}
        for r in recs:
            if r["kernel"].startswith("layer"):
                key = f"{r['kernel']}[{r['layer']}]"
                e = per_layer.setdefault(key, [0, 0.0, 0.0, r])
                e[0] += 1
                e[1] += r["ms"]
                e[2] += r["bytes"]
            e = per.setdefault(r["kernel"], [0, 0.0, 0.0])
            e[0] += 1
            e[1] += r["ms"]
            e[2] += r["bytes"]
        return per, per_layer

    def baselines(self):
        """Mean, Median, Krum (Section 6.1.1, Definitions 4 and 5) and the aggregation that also takes the server's SGD
        step (Algorithm 1), on the same candidates: one unrecorded warm-up pass, three recorded ones."""
        B, torch, w = self.B, self.torch, self.w
        x_step = w.x.clone()
        for i in range(-1, 3):
            B.profile_enable(i >= 0)
            G = self.Gs[i % self.n_buf]
            B.zeno_mean(G, out=self.out)
            B.zeno_median(G, out=self.out)
            B.zeno_aggregate_update(G, self.scores, w.b, w.gamma, x_step, x_next=x_step, want_out=False, selected=self.sel)
            if 3 <= w.m <= 128 and w.m - w.b - 2 >= 1:
                B.zeno_krum(G, w.b, out=self.out)
        torch.cuda.synchronize()
        per = {}
        for name, layer, ms, nbytes in B.profile_collect():
            e = per.setdefault(name, [0, 0.0, 0.0])
            e[0] += 1
            e[1] += ms
            e[2] += nbytes
        B.profile_enable(False)
        return {k: {"avg_ms": v[1] / v[0], "algorithmic_GBps": (v[2] / v[0]) / (v[1] / v[0]) / 1e6} for k, v in per.items()}

    def summary(self, steps, warmup, graph=False):
        """ms per step, roofline fraction of the step, and the per-launch table of one workload."""
        elapsed = self.time_steps(steps, warmup)
        ms = 1e3 * elapsed / steps
        per, per_layer = self.launches(max(3, min(steps, 10)))
        n_prof = max(3, min(steps, 10))
        w = self.w
        out = {"workload": describe(self.cfg, w), "G_row_pitch_floats": int(w.G.stride(0)) if w.m > 1 else w.d,
               "G_buffers_rotated": self.n_buf, "steps": steps, "ms_per_step": ms, "aggregations_per_s": steps / elapsed,
               "step_algorithmic_GBps": self.step_bytes / (ms * 1e-3) / 1e9,
               "step_frac_of_hbm_peak": self.step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "launches": {k: {"per_step": v[0] / n_prof, "avg_ms": v[1] / v[0],
                                "algorithmic_GBps": (v[2] / v[0]) / (v[1] / v[0]) / 1e6} for k, v in per.items()},
               "layers": layer_table(per_layer)}
        if w.m * w.d * 4 >= (1 << 30):
            out["baseline_aggregators"] = self.baselines()
        if graph:
            g_elapsed = self.time_graph(steps, warmup)
            out["graph_replay_ms_per_step"] = 1e3 * g_elapsed / steps
            out["graph_replay_aggregations_per_s"] = steps / g_elapsed
        return out


def _with_G(w, G):
    import copy
    w2 = copy.copy(w)
    w2.G = G
    return w2


def describe(cfg, w):
    return (f"config {cfg}: " + "->".join(str(v) for v in w.dims) +
            f" {w.loss}, d={w.d}, m={w.m}, b={w.b}, n_r={w.n_r}, gamma={w.gamma}, rho={w.rho}")


def layer_table(per_layer):
    return {k: {"avg_ms": v[1] / v[0], "algorithmic_GBps": v[2] / v[1] / 1e6,
                "shape": {key: v[3][key] for key in ("waves", "k_split", "k_slices", "streaming", "row_blocks", "merged", "second", "tail_candidates")}}
            for k, v in per_layer.items()}


CNN_DESC = dict(in_h=32, in_w=32, in_c=3, conv_c=[32, 32, 64, 64], conv_stride=[1, 2, 1, 2], fc_out=10, has_bias=True)


def cnn_summary(B, WL, torch, row_align, steps=100, warmup=10):
    """The shape of the paper's own experiments (Section 6: 32 x 32 x 3 images, four convolutions + one fully
    connected layer, 10 classes, m = 20, q = b = 8, n_r = 4, gamma = 0.1, rho = 5e-4; widths 32-32-64-64 and
    strides 1-2-1-2 are this benchmark's choice): zeno_score + zeno_aggregate per step.  d is 0.1 M, so the step is
    bound by the latency of its launches, not by HBM; reported as time and as matrix-core work."""
    dev = torch.device("cuda", 0)
    w = WL.make_cnn_workload("cnn_paper_shaped", 37, CNN_DESC, 20, 8, 4, 0.1, 5e-4, n_flip=8, worker_batch=16,
                             device=dev, row_align=row_align)
    mdl = B.ZenoCnnModel(w.desc, w.loss)
    ws = B.alloc_workspace(mdl, w.m, w.n_r, dev)
    scores = torch.empty(w.m, device=dev)
    out = torch.empty(w.d, device=dev)
    sel = torch.empty(w.m - w.b, dtype=torch.int32, device=dev)

    def step():
        B.zeno_score(mdl, w.x, w.G, w.features, w.gamma, w.rho, labels=w.labels, scores=scores, workspace=ws)
        B.zeno_aggregate(w.G, scores, w.b, out=out, selected=sel)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / steps
    B.profile_enable(True)
    for _ in range(5):
        step()
    torch.cuda.synchronize()
    recs = B.profile_collect(detail=True)
    B.profile_enable(False)
    per = {}
    for r in recs:
        e = per.setdefault(f"{r['kernel']}[{r['layer']}]", [0, 0.0, r["bytes"]])
        e[0] += 1
        e[1] += r["ms"]
    shapes = WL.cnn_shapes(w.desc)
    flops = 0.0
    for l, ((_, _, ci), (ho, wo, co)) in enumerate(zip(shapes[:-1], shapes[1:])):
        flops += 2.0 * w.n_r * ho * wo * 9 * ci * co * (1 + w.m * (2 if l > 0 else 1))
    ho, wo, co = shapes[-1]
    flops += 2.0 * w.n_r * ho * wo * co * w.desc["fc_out"] * (1 + 2 * w.m)
    return {"workload": f"CNN 32x32x3 -> conv {w.desc['conv_c']} strides {w.desc['conv_stride']} -> fc 10, d={w.d}, "
                        f"m={w.m}, b={w.b}, n_r={w.n_r}, gamma={w.gamma}, rho={w.rho}, fp32 forward",
            "ms_per_step": ms, "aggregations_per_s": 1e3 / ms, "matrix_core_TFLOPs": flops / (ms * 1e-3) / 1e12,
            "launches": {k: {"avg_ms": v[1] / v[0]} for k, v in per.items()}}


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

    R = Runner(B, WL, torch, a.config, a.row_align, n_r=a.n_r or None, buffers=a.buffers)
    w = R.w
    m, d, b = w.m, w.d, w.b
    g_bytes = 4 * m * d

    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.ceil(src, out=dst)   # a plain elementwise kernel: reads 4 GiB, writes 4 GiB
        torch.cuda.synchronize()
        del src, dst

    elapsed = R.time_steps(a.steps, a.warmup)
    ms_per_step = 1e3 * elapsed / a.steps

    n_prof = max(3, min(a.steps, 10))
    per, per_layer = R.launches(n_prof)
    # the baseline aggregators on the same G (Section 6.1.1, Definitions 4 and 5), and the variant of
    # the aggregation that also takes the server's SGD step (Algorithm 1), in place on a copy of x
    x_step = w.x.clone()
    for i in range(-1, 3):                             # the first pass is an unrecorded warm-up
        B.profile_enable(i >= 0)
        B.zeno_mean(R.Gs[i % R.n_buf], out=R.out)
        B.zeno_median(R.Gs[i % R.n_buf], out=R.out)
        B.zeno_aggregate_update(R.Gs[i % R.n_buf], R.scores, b, w.gamma, x_step, x_next=x_step, want_out=False,
                                selected=R.sel)
        if 3 <= m <= 128 and m - b - 2 >= 1:
            B.zeno_krum(R.Gs[i % R.n_buf], b, out=R.out)     # Krum_b (Definition 5), the paper's main baseline
    torch.cuda.synchronize()
    for name, layer, ms, nbytes in B.profile_collect():
        e = per.setdefault(name, [0, 0.0, 0.0])
        e[0] += 1
        e[1] += ms
        e[2] += nbytes
    B.profile_enable(False)
    kernels = {k: {"launches_per_step": v[0] / (3 if k in ("mean", "median", "average_update", "krum") else n_prof), "avg_ms": v[1] / v[0],
                   "algorithmic_GBps": (v[2] / v[0]) / (v[1] / v[0]) / 1e6} for k, v in per.items()}
    dom = per["layer_cand"]
    dom_avg_ms = dom[1] / dom[0]
    dom_bytes = dom[2] / dom[0]
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9

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
        "config": {"workload": describe(a.config, w),
                   "G_bytes": g_bytes, "G_row_pitch_floats": int(w.G.stride(0)), "G_buffers_rotated": R.n_buf},
        "step_algorithmic_GBps": R.step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": R.step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "layer_kernel (candidate layers, streams G)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(a.config),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_avg_ms},
        "kernels": kernels,
        "layers": layer_table(per_layer),
    }
    if not a.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, a.cpu_seconds)

    if not a.no_extras and a.config == 5 and not a.n_r:
        # the other bandwidth-bound measurements, after the headline one (not part of `value`)
        also = {}
        extra_steps = max(5, a.steps // 2)
        if a.row_align > 1:
            Rd = Runner(B, WL, torch, 5, 1, w=w)                 # the same candidates as G[m x d], ld = d
            also["config5_dense_rows"] = Rd.summary(extra_steps, 2)
            del Rd
        del R
        torch.cuda.empty_cache()
        also["config4"] = Runner(B, WL, torch, 4, a.row_align).summary(extra_steps, 2)
        torch.cuda.empty_cache()
        for cfg in (3, 2, 1):
            also[f"config{cfg}"] = Runner(B, WL, torch, cfg, a.row_align).summary(200, 20, graph=True)
        also["cnn_paper_shaped"] = cnn_summary(B, WL, torch, a.row_align)
        result["also"] = also
    print(json.dumps(result))


if __name__ == "__main__":
    main()
