#!/usr/bin/env python3
"""Benchmark of the IDKM hot path on one MI355X.

One "step" = one pass of the whole hot path over one layer: idkm_forward (soft k-means to
convergence + evaluation at C*) followed by idkm_backward (implicit fixed-point solve).
Headline workload: the 3x3x512x512 ResNet18 layer as scalars (m = 2,359,296, d = 1, k = 4),
synthetic Kaiming-normal weights, squared-distance energy.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--dist sql2|l2] [--path auto|stream|persistent]
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

# MI355X: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz full-rate VALU lane-operations per second
# (an FMA counts once; packed-fp32 forms are disabled in this build, so this is the issue peak).
PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
PEAK_HBM = 8.0e12
TRANS_COST = 4  # a transcendental (exp2, rcp, sqrt, rsq) occupies four full-rate issue slots


def fwd_lane_ops_per_vector(k: int, d: int, dist: int) -> int:
    """Algorithmic lane-cycles of one forward evaluation per weight vector:
    k (3d+5) full-rate operations (2d distance, 1 min, 1 logit, 1 sum, 1 normalise, d+1 accumulate)
    plus k+1 transcendentals (k exp2, 1 reciprocal; k more square roots for the plain norm with d > 1)."""
    trans = k + 1 + (k if (dist == 0 and d > 1) else 0)
    return k * (3 * d + 5) + TRANS_COST * trans


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4"])
    ap.add_argument("--dist", default="sql2", choices=["sql2", "l2"])
    ap.add_argument("--path", default="auto", choices=["auto", "stream", "persistent"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--bwd-tol", type=float, default=1e-6)
    ap.add_argument("--bwd-max-iter", type=int, default=2000)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2312_07759_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dist = wl.DIST_SQL2 if args.dist == "sql2" else wl.DIST_L2
    p = wl.make_problem(args.workload, dist)
    cfg = p.cfg
    ctx = binding.Context(0)
    ctx.set_path({"auto": binding.PATH_AUTO, "stream": binding.PATH_STREAM, "persistent": binding.PATH_PERSISTENT}[args.path])
    W = torch.from_numpy(p.W).cuda()
    C0 = torch.from_numpy(p.C0).cuda()
    if p.G is not None:
        G = torch.from_numpy(p.G).cuda()
    else:
        G = torch.from_numpy(wl.draw_weights(cfg.m * cfg.d, 1e-4, cfg.g_seed).reshape(cfg.m, cfg.d)).cuda()
    torch.cuda.synchronize()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(timing=None):
        e = [ev() for _ in range(4)] if timing is not None else None
        if e:
            e[0].record()
        f = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_A=False, want_Wq=True)
        if e:
            e[1].record()
        b = ctx.backward(G, binding.BWD_IMPLICIT, tol=args.bwd_tol, max_iter=args.bwd_max_iter, alpha=1.0)
        if e:
            e[2].record()
        j = ctx.backward(G, binding.BWD_JFB)
        if e:
            e[3].record()
            timing.append((e, f["info"], b["info"]))
        return f, b, j

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly K steps of forward + implicit backward (the JFB call is timed separately below)
    t0 = time.perf_counter()
    infos = []
    for _ in range(args.steps):
        f = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_A=False, want_Wq=True)
        b = ctx.backward(G, binding.BWD_IMPLICIT, tol=args.bwd_tol, max_iter=args.bwd_max_iter, alpha=1.0)
        infos.append((f["info"], b["info"]))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-phase timing with events on the stream the kernels run on
    timing = []
    nrep = max(3, min(args.steps, 10))
    for _ in range(nrep):
        step(timing)
    torch.cuda.synchronize()
    fwd_ms = float(np.median([e[0].elapsed_time(e[1]) for e, _, _ in timing]))
    bwd_ms = float(np.median([e[1].elapsed_time(e[2]) for e, _, _ in timing]))
    jfb_ms = float(np.median([e[2].elapsed_time(e[3]) for e, _, _ in timing]))
    finfo, binfo = timing[-1][1], timing[-1][2]
    fwd_evals = finfo.iters + 1  # + the evaluation at C*
    iters_per_s = finfo.iters / (fwd_ms * 1e-3)

    ops_vec = fwd_lane_ops_per_vector(cfg.k, cfg.d, dist)
    per_eval_s = fwd_ms * 1e-3 / fwd_evals
    alu_achieved = ops_vec * cfg.m / per_eval_s
    hbm_eff = 4.0 * cfg.m * cfg.d / per_eval_s
    roofline = {
        "bound": "alu", "kernel": "forward evaluation of F (E-step + M-step over all m vectors)",
        "achieved": alu_achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
        "frac": alu_achieved / PEAK_LANE_OPS, "traffic": None,
        "lane_ops_per_vector": ops_vec, "evaluations_per_launch": fwd_evals if finfo.path == 2 else 1,
        "avg_eval_us": per_eval_s * 1e6,
        "hbm_effective_GBps": hbm_eff / 1e9, "hbm_effective_frac": hbm_eff / PEAK_HBM,
    }

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import idkm_oracle as orc
        try:
            from threadpoolctl import threadpool_limits
            limiter = threadpool_limits(limits=1)
        except Exception:  # pragma: no cover
            limiter = None
        n_eval = 0
        C = p.C0.astype(np.float64)
        Wh = p.W.astype(np.float64)
        tc0 = time.perf_counter()
        while True:
            C = orc.F(C, Wh, p.tau, dist)
            n_eval += 1
            el = time.perf_counter() - tc0
            if el > 12.0 or n_eval >= 40:
                break
        if limiter is not None:
            limiter.restore_original_limits() if hasattr(limiter, "restore_original_limits") else None
        cpu = {"value": n_eval / el, "unit": "iters/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_eval} evaluations of F (float64 numpy) on the full {cfg.name} tensor, m={cfg.m}, k={cfg.k}, d={cfg.d}"}

    out = {
        "metric": "soft-k-means forward iters/s (implicit-backward and JFB ms per layer alongside)",
        "value": iters_per_s, "unit": "iters/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: m={cfg.m} d={cfg.d} k={cfg.k} tau={cfg.tau} tol={cfg.tol} "
                               f"max_iter={cfg.max_iter} dist={wl.DIST_NAMES[dist]} ({cfg.note})",
                   "path": {1: "stream", 2: "persistent"}.get(finfo.path, str(finfo.path))},
        "forward": {"ms": fwd_ms, "iters": finfo.iters, "converged": finfo.converged, "residual": finfo.residual},
        "implicit_backward": {"ms": bwd_ms, "passes": binfo.iters, "converged": binfo.converged,
                              "tol": args.bwd_tol},
        "jfb_backward": {"ms": jfb_ms},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
