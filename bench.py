#!/usr/bin/env python3
"""Benchmark of the IDKM hot path on one MI355X.

One "step" = one pass of the whole hot path over one layer: idkm_forward (soft k-means to
convergence + the evaluation at C*) followed by idkm_backward (implicit fixed-point solve).
Headline workload: the 3x3x512x512 ResNet18 layer as scalars (m = 2,359,296, d = 1, k = 4),
synthetic Kaiming-normal weights, squared-distance energy.  Prints ONE JSON line; the other
configurations ride along under "others" (forward / implicit / JFB times and roofline fraction).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--dist sql2|l2]
                  [--path auto|stream|persistent] [--no-others] [--no-cpu-baseline]
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

# MI355X: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz full-rate VALU lane-operations per second.
# An FMA counts once; packed-fp32 forms are disabled in this build, so this is the issue peak
# (the data-sheet 157.3 TFLOP/s fp32 = 2 flops per FMA x 2 packed lanes x this figure).
PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
PEAK_HBM = 8.0e12
# A transcendental (exp2, rcp, sqrt, rsq) occupies TWO full-rate issue slots on this part: idkm_calibrate measures
# 16.4 T v_exp_f32/s against 33.4 T v_fma_f32/s (the live figures are reported under roofline.ceilings).
TRANS_COST = 2


def fwd_lane_ops_per_vector(k: int, d: int, dist: int) -> int:
    """Algorithmic lane-cycles of one evaluation of F per weight vector:
    k (3d+5) full-rate operations (2d distance, 1 min, 1 logit, 1 sum, 1 normalise, d+1 accumulate)
    plus k+1 transcendentals (k exp2, 1 reciprocal; k more square roots for the plain norm with d > 1), each counted
    with its measured cost of two issue slots."""
    trans = k + 1 + (k if (dist == 0 and d > 1) else 0)
    return k * (3 * d + 5) + TRANS_COST * trans


def bwd_lane_ops_per_vector(k: int, d: int, dist: int) -> int:
    """Algorithmic lane-cycles of one (dF/dC)^T pass per weight vector: about k (5d+9) full-rate operations (the
    E-step of the forward evaluation plus beta, its row mean, gamma and the k d accumulations) and the same k+1
    transcendentals, each at two issue slots."""
    trans = k + 1 + (k if (dist == 0 and d > 1) else 0)
    return k * (5 * d + 9) + TRANS_COST * trans


def matrix_core_lane_cycles_per_vector(k: int, dist: int) -> int:
    """The same count for the shapes whose forward loop runs on the matrix cores (d = 4, 17 <= k <= 256, persistent
    path): per (vector, codeword) pair 8 float32 multiply-adds on the matrix cores (4 of the energy product, 4 of
    the first moments) and, squared energy, 4 vector issue slots (exp2 = 2, row sum, mass); the plain norm adds the
    codeword's norm, a square root (2), the row minimum and its subtraction: 9.  A SIMD retires 32 matrix
    multiply-adds or 16 lane operations per cycle and -- measured, idkm_calibrate kinds 6 and 7 -- never both at
    once, so a matrix multiply-add is half a lane-cycle: 8/2 + 4 = 8 (resp. 13) lane-cycles per pair, plus the
    reciprocal of the row sum."""
    return k * (8 if dist == 1 else 13) + TRANS_COST


def measure_dense(ctx, binding, torch, np, G, reps):
    """Median event time (ms) of the dense (explicit-Jacobian) backward, or None where it is not offered."""
    ts = []
    try:
        for _ in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ctx.backward(G, binding.BWD_DENSE)
            e1.record()
            ts.append((e0, e1))
        torch.cuda.synchronize()
    except binding.IdkmError:
        return None
    return float(np.median([a.elapsed_time(b) for a, b in ts[1:]]))


def measure_gmres(ctx, binding, torch, np, G, reps, tol, max_iter):
    """Median event time (ms) and the last info of the minimal-residual (Krylov) backward."""
    ts = []
    info = None
    for _ in range(reps + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        info = ctx.backward(G, binding.BWD_GMRES, tol=tol, max_iter=max_iter)["info"]
        e1.record()
        ts.append((e0, e1))
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in ts[1:]])), info


def measure(ctx, binding, torch, np, p, dist, W, C0, G, reps, bwd_tol, bwd_max_iter):
    """Median event times (ms) of forward, implicit backward and JFB backward over `reps` runs."""
    recs = []
    kern = {"fwd": [], "bwd": [], "jfb": []}

    def kernel_ms(key):
        # the launch itself, bracketed by events the library records on this stream right around it (persistent path)
        try:
            kern[key].append(ctx.last_kernel_ms())
        except binding.IdkmError:
            pass

    # outputs are allocated once, as a training loop would keep them
    fo = {"C": torch.empty_like(C0), "Wq": torch.empty_like(W)}
    dW = torch.empty_like(G)
    ctx.set_kernel_timing(True)
    for _ in range(reps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record()
        f = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_A=False, want_Wq=True, out=fo)
        e[1].record()
        kernel_ms("fwd")
        b = ctx.backward(G, binding.BWD_IMPLICIT, tol=bwd_tol, max_iter=bwd_max_iter, alpha=1.0, out=dW)
        e[2].record()
        kernel_ms("bwd")
        ctx.backward(G, binding.BWD_JFB, out=dW)
        e[3].record()
        kernel_ms("jfb")
        recs.append((e, f["info"], b["info"]))
    torch.cuda.synchronize()
    ctx.set_kernel_timing(False)
    fwd = float(np.median([e[0].elapsed_time(e[1]) for e, _, _ in recs]))
    bwd = float(np.median([e[1].elapsed_time(e[2]) for e, _, _ in recs]))
    jfb = float(np.median([e[2].elapsed_time(e[3]) for e, _, _ in recs]))
    measure.kernel_ms = {k: (float(np.median(v)) if len(v) == reps else None) for k, v in kern.items()}
    return fwd, bwd, jfb, recs[-1][1], recs[-1][2]


def roofline_of(cfg, dist, fwd_ms, finfo, kernel_ms=None):
    """fwd_ms: event time of the whole idkm_forward call; kernel_ms: event time of its one persistent launch (None on
    the stream path, where a solve is many launches and the call is what can be timed)."""
    evals = finfo.iters + 1  # + the evaluation at C*
    call_per_eval = fwd_ms * 1e-3 / evals
    per_eval = (kernel_ms if kernel_ms else fwd_ms) * 1e-3 / evals
    valu_ops = fwd_lane_ops_per_vector(cfg.k, cfg.d, dist)
    matrix = cfg.d == 4 and 17 <= cfg.k <= 256 and finfo.path == 2
    ops = matrix_core_lane_cycles_per_vector(cfg.k, dist) if matrix else valu_ops
    alu = ops * cfg.m / per_eval
    hbm = 4.0 * cfg.m * cfg.d / per_eval
    out = {
        "bound": "alu", "kernel": "forward solve: evaluations of F (E-step + M-step over all m vectors)",
        "achieved": alu / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s", "frac": alu / PEAK_LANE_OPS,
        "traffic": None, "lane_ops_per_vector": ops,
        "evaluations_per_launch": evals if finfo.path == 2 else 1, "avg_eval_us": per_eval * 1e6,
        "hbm_effective_GBps": hbm / 1e9, "hbm_effective_frac": hbm / PEAK_HBM,
        "timed": ("the forward solve's one kernel launch, HIP events recorded by the library on the launch stream right "
                  "before and after it" if kernel_ms else "the whole idkm_forward call (one launch per pass)"),
        "kernel_ms": kernel_ms, "call_ms": fwd_ms, "frac_over_the_call": ops * cfg.m / call_per_eval / PEAK_LANE_OPS,
    }
    if matrix:
        out["note"] = ("forward loop on the matrix cores: a float32 matrix multiply-add counts as half a lane-cycle "
                       "(32 per cycle and SIMD, not concurrent with the vector ALU)")
        out["frac_of_vector_alu_bound"] = valu_ops * cfg.m / per_eval / PEAK_LANE_OPS
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "P16", "XL"])
    ap.add_argument("--dist", default="sql2", choices=["sql2", "l2"])
    ap.add_argument("--path", default="auto", choices=["auto", "stream", "persistent"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true")
    ap.add_argument("--bwd-tol", type=float, default=1e-6)
    ap.add_argument("--bwd-max-iter", type=int, default=2000)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain elementwise copy of 64 Mi floats (reads 256 MiB, writes 256 MiB) three "
                         "times, as the known-size reference for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")
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
    path_id = {"auto": binding.PATH_AUTO, "stream": binding.PATH_STREAM, "persistent": binding.PATH_PERSISTENT}[args.path]
    ctx = binding.Context(0)
    ctx.set_path(path_id)

    def load(name, dist):
        p = wl.make_problem(name, dist)
        cfg = p.cfg
        W = torch.from_numpy(p.W).cuda()
        C0 = torch.from_numpy(p.C0).cuda()
        g = p.G if p.G is not None else wl.draw_weights(cfg.m * cfg.d, 1e-4, cfg.g_seed).reshape(cfg.m, cfg.d)
        return p, W, C0, torch.from_numpy(g).cuda()

    if args.calib_copy:
        x = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y

    dist = wl.DIST_SQL2 if args.dist == "sql2" else wl.DIST_L2
    p, W, C0, G = load(args.workload, dist)
    cfg = p.cfg
    fo = {"C": torch.empty_like(C0), "Wq": torch.empty_like(W)}  # outputs allocated once, as a training loop keeps them
    dWo = torch.empty_like(G)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_A=False, want_Wq=True, out=fo)
        ctx.backward(G, binding.BWD_IMPLICIT, tol=args.bwd_tol, max_iter=args.bwd_max_iter, alpha=1.0, out=dWo)
    torch.cuda.synchronize()
    # timed region: exactly K steps of forward + implicit backward, inputs resident in HBM
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_A=False, want_Wq=True, out=fo)
        ctx.backward(G, binding.BWD_IMPLICIT, tol=args.bwd_tol, max_iter=args.bwd_max_iter, alpha=1.0, out=dWo)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-phase times with events on the stream the kernels run on (the binding passes torch's current stream)
    fwd_ms, bwd_ms, jfb_ms, finfo, binfo = measure(ctx, binding, torch, np, p, dist, W, C0, G,
                                                   max(5, min(args.steps, 20)), args.bwd_tol, args.bwd_max_iter)
    # the ceilings themselves, measured on this device (the roofline's peak stays the published figure)
    fma_rate = ctx.calibrate(0)
    exp_rate = ctx.calibrate(1)
    big = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    read_rate = ctx.calibrate(2, big)
    del big
    dense_ms = measure_dense(ctx, binding, torch, np, G, 5)
    gm_ms, gm_info = measure_gmres(ctx, binding, torch, np, G, 5, args.bwd_tol, args.bwd_max_iter)
    kms = dict(measure.kernel_ms)
    roofline = roofline_of(cfg, dist, fwd_ms, finfo, kms.get("fwd"))
    # the (dF/dC)^T passes of the implicit backward (Eq. "backiter"): the JFB call is the same launch without them
    # (one pass for v, one for dL/dW), so their time is the difference of the two calls
    roofline_backward = None
    if binfo.iters > 0:
        bops = bwd_lane_ops_per_vector(cfg.k, cfg.d, dist)
        use_kernel = bool(kms.get("bwd") and kms.get("jfb"))
        b_ms, j_ms = (kms["bwd"], kms["jfb"]) if use_kernel else (bwd_ms, jfb_ms)
        per_pass = max(b_ms - j_ms, 1e-9) * 1e-3 / binfo.iters
        roofline_backward = {
            "bound": "alu", "kernel": "implicit backward: (dF/dC)^T passes of the averaged iteration (E-step recomputed in every pass)",
            "achieved": bops * cfg.m / per_pass / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
            "frac": bops * cfg.m / per_pass / PEAK_LANE_OPS, "lane_ops_per_vector": bops, "passes": binfo.iters,
            "us_per_pass": per_pass * 1e6, "implicit_ms": b_ms, "jfb_ms": j_ms,
            "timed": "kernel launches (library-recorded events)" if use_kernel else "whole calls",
            "note": "time per pass = (implicit launch - JFB launch) / passes; lane-ops per vector = k (5d+9) + 2 (k+1)"}
        if cfg.d == 4 and 17 <= cfg.k <= 256 and binfo.path == 2:
            roofline_backward["note"] += ("; this shape runs the passes on the matrix cores, so the fraction is against "
                                          "the vector-ALU count and can exceed what the vector ALU alone could reach")
    mfma_rate, mfma_mixed, mfma4_rate = ctx.calibrate(6), ctx.calibrate(7), ctx.calibrate(8)
    mfma_mixed_4w, mfma_mixed_8w, mfma_rate_4w = ctx.calibrate(9), ctx.calibrate(10), ctx.calibrate(11)
    roofline["ceilings"] = {"fma_Tlane_ops": fma_rate / 1e12, "exp_T_per_s": exp_rate / 1e12,
                            "mfma_f32_16x16x4_Tmac_per_s": mfma_rate / 1e12,
                            "mfma_f32_16x16x4_Tmac_per_s_with_8_fma_each": mfma_mixed / 1e12,
                            "mfma_f32_4x4x1_Tmac_per_s": mfma4_rate / 1e12,
                            "mfma_f32_16x16x4_Tmac_per_s_4_waves_per_simd": mfma_rate_4w / 1e12,
                            "mfma_f32_16x16x4_Tmac_per_s_with_8_fma_each_4_waves_per_simd": mfma_mixed_4w / 1e12,
                            "mfma_f32_16x16x4_Tmac_per_s_with_8_fma_each_8_waves_per_simd": mfma_mixed_8w / 1e12,
                            "slots_per_transcendental": fma_rate / exp_rate, "stream_read_GBps": read_rate / 1e9,
                            "frac_of_measured_fma_rate": roofline["achieved"] * 1e12 / fma_rate,
                            "note": "idkm_calibrate on this device: v_fma_f32 chains, v_exp_f32 chains, float32 matrix "
                                    "instructions alone and with vector FMAs between them, 256 MiB streaming read"}
    # HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command
    # (counters cannot be read from inside the process; the summary under profiles/ gives the commands)
    tpath = os.path.join(ROOT, "profiles", f"traffic_{cfg.name}_{wl.DIST_NAMES[dist]}.json")
    if finfo.path == 2 and os.path.exists(tpath):
        with open(tpath) as f:
            t = json.load(f)
        lib_version = int(binding.load_library().idkm_version())
        roofline["traffic"] = {"fetch_bytes": t["fetch_bytes"], "write_bytes": t["write_bytes"],
                               "algorithmic_bytes": 8 * cfg.m * cfg.d, "per": t["per"], "source": t["source"],
                               "measured_with_library_version": t.get("library_version"),
                               "measured_at_commit": t.get("commit"),
                               "stale": t.get("library_version") != lib_version}

    others = None
    if not args.no_others:
        others = []
        for name, dd in (("C1", 1), ("C1", 0), ("C2", 1), ("C2", 0), ("C3", 0), ("C4", 1), ("C4", 0), ("P16", 1),
                         ("P16", 0), ("XL", 1)):
            del W, C0, G
            q, W, C0, G = load(name, dd)
            measure(ctx, binding, torch, np, q, dd, W, C0, G, 1, args.bwd_tol, 300)
            f_ms, b_ms, j_ms, fi, bi = measure(ctx, binding, torch, np, q, dd, W, C0, G, 3, args.bwd_tol, 300)
            r = roofline_of(q.cfg, dd, f_ms, fi, measure.kernel_ms.get("fwd"))
            d_ms = measure_dense(ctx, binding, torch, np, G, 3)
            g_ms, gi = measure_gmres(ctx, binding, torch, np, G, 2, args.bwd_tol, 300)
            others.append({"dense_ms": None if d_ms is None else round(d_ms, 4), "workload": name, "dist": wl.DIST_NAMES[dd], "m": q.cfg.m, "d": q.cfg.d, "k": q.cfg.k,
                           "path": {1: "stream", 2: "persistent"}.get(fi.path), "fwd_ms": round(f_ms, 4),
                           "fwd_iters": fi.iters, "fwd_converged": fi.converged,
                           "fwd_iters_per_s": round(fi.iters / (f_ms * 1e-3), 1),
                           "implicit_ms": round(b_ms, 4), "implicit_passes": bi.iters,
                           "implicit_converged": bi.converged, "jfb_ms": round(j_ms, 4),
                           "gmres_ms": round(g_ms, 4), "gmres_passes": gi.iters, "gmres_converged": gi.converged,
                           "gmres_residual": gi.residual,
                           "alu_frac": round(r["frac"], 4), "avg_eval_us": round(r["avg_eval_us"], 3)})

        # the whole-network sweep: 21 ResNet18 tensors, each quantised independently at k = 2 and k = 4 (d = 1)
        for dd in (1, 0):
            tot = {"fwd_ms": 0.0, "implicit_ms": 0.0, "jfb_ms": 0.0, "fwd_iters": 0, "implicit_passes": 0,
                   "unconverged_fwd": 0, "unconverged_bwd": 0, "weights": 0, "layers": 0}
            bt = {"fwd_ms": 0.0, "implicit_ms": 0.0, "jfb_ms": 0.0, "dense_ms": 0.0, "launches_fwd": 0}
            for kk in (2, 4):
                held = []
                for ti in range(len(wl.RESNET18_TENSORS)):
                    q = wl.make_problem(wl.sweep_config(ti, kk, dd), dd)
                    Wt, Ct, Gt = (torch.from_numpy(x).cuda() for x in (q.W, q.C0, q.G))
                    held.append((q, Wt, Ct, Gt))
                    measure(ctx, binding, torch, np, q, dd, Wt, Ct, Gt, 1, args.bwd_tol, 2000)
                    f_ms, b_ms, j_ms, fi, bi = measure(ctx, binding, torch, np, q, dd, Wt, Ct, Gt, 2, args.bwd_tol, 2000)
                    tot["fwd_ms"] += f_ms
                    tot["implicit_ms"] += b_ms
                    tot["jfb_ms"] += j_ms
                    tot["fwd_iters"] += fi.iters
                    tot["implicit_passes"] += bi.iters
                    tot["unconverged_fwd"] += 0 if fi.converged else 1
                    tot["unconverged_bwd"] += 0 if bi.converged else 1
                    tot["weights"] += q.cfg.m
                    tot["layers"] += 1
                # the same 21 tensors through the batched entry points: one call for all layers
                batch = binding.Batch(len(held))
                pairs = [(Wt, Ct) for _, Wt, Ct, _ in held]
                taus = [q.tau for q, _, _, _ in held]
                Gs = [Gt for _, _, _, Gt in held]
                q0 = held[0][0]
                for rep in range(3):  # the first repetition warms up
                    ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
                    ev[0].record()
                    batch.forward(pairs, taus, q0.tol, q0.max_iter, dd, want_Wq=True)
                    ev[1].record()
                    batch.backward(Gs, binding.BWD_IMPLICIT, tol=args.bwd_tol, max_iter=2000, alpha=1.0)
                    ev[2].record()
                    batch.backward(Gs, binding.BWD_JFB)
                    ev[3].record()
                    batch.backward(Gs, binding.BWD_DENSE)
                    ev[4].record()
                    torch.cuda.synchronize()
                    if rep:
                        bt["dense_ms"] += ev[3].elapsed_time(ev[4]) / 2
                        bt["fwd_ms"] += ev[0].elapsed_time(ev[1]) / 2
                        bt["implicit_ms"] += ev[1].elapsed_time(ev[2]) / 2
                        bt["jfb_ms"] += ev[2].elapsed_time(ev[3]) / 2
                batch.forward(pairs, taus, q0.tol, q0.max_iter, dd, want_Wq=True)
                bt["launches_fwd"] += batch.launches()
                batch.close()
                del held, pairs, Gs
            others.append({"workload": "C5 (21 ResNet18 tensors x k in {2,4}, one call per tensor)",
                           "dist": wl.DIST_NAMES[dd], **{a: (round(b, 3) if isinstance(b, float) else b) for a, b in tot.items()},
                           "fwd_iters_per_s": round(tot["fwd_iters"] / (tot["fwd_ms"] * 1e-3), 1)})
            others.append({"workload": "C5 (21 ResNet18 tensors x k in {2,4}, one batched call per k)",
                           "dist": wl.DIST_NAMES[dd], **{a: (round(b, 3) if isinstance(b, float) else b) for a, b in bt.items()},
                           "fwd_iters": tot["fwd_iters"], "weights": tot["weights"], "layers": tot["layers"],
                           "fwd_iters_per_s": round(tot["fwd_iters"] / (bt["fwd_ms"] * 1e-3), 1)})

    cpu = None
    cpu_all = None
    if not args.no_cpu_baseline:
        from oracle import idkm_oracle as orc
        limiter = None
        try:
            from threadpoolctl import threadpool_limits
            limiter = threadpool_limits(limits=1)
        except Exception:  # pragma: no cover
            pass
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
            limiter.unregister() if hasattr(limiter, "unregister") else None
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                for line in f:
                    if line.startswith("model name"):
                        cpu_model = line.split(":", 1)[1].strip()
                        break
        except OSError:  # pragma: no cover
            pass
        cpu = {"value": n_eval / el, "unit": "iters/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_eval} evaluations of F (float64 numpy oracle, BLAS pinned to one thread) on the full "
                         f"{cfg.name} tensor, m={cfg.m}, k={cfg.k}, d={cfg.d}",
               "cpu_model": cpu_model, "host_cores_visible": os.cpu_count()}
        # all host cores: the numpy oracle is single-threaded by nature, so the cores are filled with independent
        # copies of the same evaluation (as the layers of a network would be), one process each, none touching the GPU
        import subprocess
        workers = max(1, min(16, os.cpu_count() or 1))
        code = ("import sys,time,numpy as np\n"
                "sys.path.insert(0, %r)\n"
                "from oracle import idkm_oracle as orc\n"
                "from paper_2312_07759_amd import workloads as wl\n"
                "p = wl.make_problem(%r, %d)\n"
                "C = p.C0.astype(np.float64); W = p.W.astype(np.float64)\n"
                "print('ready', flush=True); sys.stdin.readline()\n"
                "t0 = time.perf_counter(); n = 0\n"
                "while True:\n"
                "    C = orc.F(C, W, p.tau, %d); n += 1\n"
                "    if time.perf_counter() - t0 > 8.0 or n >= 40: break\n"
                "print(n, time.perf_counter() - t0, flush=True)\n") % (ROOT, cfg.name, dist, dist)
        env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1",
                   HIP_VISIBLE_DEVICES="", ROCR_VISIBLE_DEVICES="")
        procs = [subprocess.Popen([sys.executable, "-c", code], stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True,
                                  env=env) for _ in range(workers)]
        try:
            for q in procs:  # every worker has drawn its inputs before any of them starts the clock
                q.stdout.readline()
            for q in procs:
                q.stdin.write("go\n")
                q.stdin.flush()
            done = [q.stdout.readline().split() for q in procs]
            total = sum(int(x[0]) for x in done)
            longest = max(float(x[1]) for x in done)
            cpu_all = {"value": total / longest, "unit": "iters/s", "cores": workers, "kind": "oracle",
                       "sample": f"{workers} processes side by side, each {done[0][0]} evaluations of F on the full {cfg.name} "
                                 f"tensor (the numpy oracle is single-threaded; independent copies fill the cores)",
                       "cpu_model": cpu_model}
        except Exception as e:  # pragma: no cover
            cpu_all = {"error": repr(e)}
        finally:
            for q in procs:
                try:
                    q.stdin.close()
                    q.wait(timeout=60)
                except Exception:  # pragma: no cover
                    q.kill()

    out = {
        "metric": "soft-k-means forward iters/s (implicit-backward and JFB ms per layer alongside)",
        "value": finfo.iters / (fwd_ms * 1e-3), "unit": "iters/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: m={cfg.m} d={cfg.d} k={cfg.k} tau={cfg.tau} tol={cfg.tol} "
                               f"max_iter={cfg.max_iter} dist={wl.DIST_NAMES[dist]} ({cfg.note})",
                   "path": {1: "stream", 2: "persistent"}.get(finfo.path, str(finfo.path))},
        "forward": {"ms": fwd_ms, "iters": finfo.iters, "converged": finfo.converged, "residual": finfo.residual},
        "implicit_backward": {"ms": bwd_ms, "passes": binfo.iters, "converged": binfo.converged,
                              "tol": args.bwd_tol},
        "jfb_backward": {"ms": jfb_ms},
        "gmres_backward": {"ms": gm_ms, "passes": gm_info.iters, "converged": gm_info.converged, "tol": args.bwd_tol,
                           "path": {1: "stream", 2: "persistent"}.get(gm_info.path),
                           "note": "restarted GMRES on (I - dF/dC*)^T g = v, one pass over W per basis vector"},
        "dense_backward": {"ms": dense_ms, "note": "explicit k d x k d Jacobian in one pass + direct solve (2 passes over W)"},
        "roofline": roofline,
        "roofline_backward": roofline_backward,
        "cpu_baseline": cpu,
        "cpu_baseline_all_cores": cpu_all,
        "library_version": int(binding.load_library().idkm_version()),
        "others": others,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
