#!/usr/bin/env python3
"""Writes the full-size expected values under tests/golden/ from the CPU oracle alone.

The paper prints no worked numeric example, so nothing here is the paper's: every stored number is
computed by oracle/idkm_oracle.py (numpy float64) on the seeded inputs of
paper_2312_07759_amd/workloads.py.  The HIP path is never imported or run.  The full-size oracle
runs take minutes (a forward solve of the 3x3x256x256 layer is ~100 s), which is why they are
stored instead of being recomputed inside the GPU tests.

  python tests/golden/make_golden.py C2 C3 C4 P16 C5 C4cap P16cap     (any subset; default: all)

C4cap / P16cap run the configs that end at their iteration cap all the way to it (200 evaluations of F at
k = 256 are about an hour and a half of numpy) and then take an averaged-iteration backward of a fixed number
of passes; "C4cap:L2" or "C4cap:SQL2" runs one energy only, so that the two can run side by side.
"""
from __future__ import annotations

import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

from oracle import idkm_oracle as orc  # noqa: E402
from paper_2312_07759_amd import workloads as wl  # noqa: E402

NOTE = ("written by tests/golden/make_golden.py from oracle/idkm_oracle.py only (float64); "
        "the paper (arXiv 2312.07759) prints no worked example")
N_SAMPLE = 256


def sample_rows(m, seed, n=N_SAMPLE):
    return np.sort(np.random.default_rng(seed).choice(m, size=min(n, m), replace=False))


def dump(rec, out):
    """JSON with 12 significant digits (the GPU tolerances are 1e-4 / 1e-3)."""
    def rnd(x):
        if isinstance(x, float):
            return float("%.12g" % x)
        if isinstance(x, list):
            return [rnd(v) for v in x]
        if isinstance(x, dict):
            return {k: rnd(v) for k, v in x.items()}
        return x
    with open(out, "w") as f:
        json.dump(rnd(rec), f, separators=(",", ":"))




def solved_layer(name, dist, out):
    """Forward to the config's stop rule, then backward (dense solve of the implicit system, and JFB)."""
    p = wl.make_problem(name, dist)
    t0 = time.time()
    fw = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, p.max_iter, dist)
    C = fw["C"]
    idx = sample_rows(p.cfg.m, 77)
    rec = dict(note=NOTE, config=name, dist=dist, m=p.cfg.m, d=p.cfg.d, k=p.cfg.k, tau=p.tau, tol=p.tol,
               max_iter=p.max_iter, iters=fw["iters"], converged=fw["converged"], residual=fw["residual"],
               C=C.tolist(), sample_rows=idx.tolist())
    rec["Wq_rows"] = orc.soft_quantize(p.W[idx], C, p.tau, dist).tolist()
    rec["assign_rows_at_oracle_C"] = orc.hard_assign_f32(p.W[idx], C.astype(np.float32)).tolist()
    A = orc.attention(p.W, C, p.tau, dist)
    Fv, n = orc.mstep(A, p.W, C)
    rec["n"] = n.tolist()
    del A
    G = p.G
    # full backward needs all rows (v and the masses are sums over rows); only sampled rows of dW are stored
    dense = orc.backward(p.W, C, p.tau, dist, G, "dense")
    jfb = orc.backward(p.W, C, p.tau, dist, G, "jfb")
    rec["v"] = dense["v"].tolist()
    rec["g_dense"] = dense["g"].tolist()
    rec["dW_implicit_rows"] = dense["dW"][idx].tolist()
    rec["dW_jfb_rows"] = jfb["dW"][idx].tolist()
    rec["dW_implicit_norm"] = float(np.linalg.norm(dense["dW"]))
    rec["dW_jfb_norm"] = float(np.linalg.norm(jfb["dW"]))
    rec["dW_implicit_colsum"] = dense["dW"].sum(0).tolist()
    rec["G_colsum"] = G.astype(np.float64).sum(0).tolist()
    # the averaged iteration of Sec. 4.2 held to a fixed number of passes (tol = 0): comparable pass by pass whether
    # or not it would meet its stop rule; and the spectral radius of dF/dC*, which says whether it ever would
    it40 = orc.backward(p.W, C, p.tau, dist, G, "implicit", tol=0.0, max_iter=40, alpha=1.0)
    rec["implicit40"] = dict(iters=it40["iters"], alpha=it40["alpha"], residual=it40["residual"], g=it40["g"].tolist(),
                             dW_rows=it40["dW"][idx].tolist(), dW_norm=float(np.linalg.norm(it40["dW"])),
                             dW_absmax=float(np.abs(it40["dW"]).max()))
    rec["rho"] = float(np.abs(np.linalg.eigvals(orc.jacobian_C(C, p.W, p.tau, dist))).max())
    rec["oracle_seconds"] = round(time.time() - t0, 1)
    dump(rec, out)
    print(name, dist, "iters", fw["iters"], "conv", fw["converged"], "%.0fs" % (time.time() - t0), flush=True)


def stepwise_layer(name, dist, out, steps):
    """For the configs that do not converge within their cap (k = 256; k = 16 with d = 4): one evaluation of F and one
    (dF/dC)^T pass at C0, the trajectory after `steps` evaluations, and the JFB gradient there."""
    p = wl.make_problem(name, dist)
    t0 = time.time()
    k, d = p.cfg.k, p.cfg.d
    idx = sample_rows(p.cfg.m, 78, 64)
    A = orc.attention(p.W, p.C0, p.tau, dist)
    F0, n0 = orc.mstep(A, p.W, p.C0)
    del A
    g = np.random.default_rng(79).standard_normal((k, d)).astype(np.float32)
    u0 = orc.vjp_F(p.C0, p.W, p.tau, dist, g)[0]
    fw = orc.soft_kmeans(p.W, p.C0, p.tau, 0.0, steps, dist)
    C = fw["C"]
    rec = dict(note=NOTE, config=name, dist=dist, m=p.cfg.m, d=d, k=k, tau=p.tau, steps=steps,
               F_at_C0=F0.tolist(), n_at_C0=n0.tolist(), g=g.tolist(), JCTg_at_C0=u0.tolist(),
               C_after_steps=C.tolist(), residual_after_steps=fw["residual"], sample_rows=idx.tolist())
    rec["Wq_rows"] = orc.soft_quantize(p.W[idx], C, p.tau, dist).tolist()
    jfb = orc.backward(p.W, C, p.tau, dist, p.G, "jfb")
    rec["v"] = jfb["v"].tolist()
    rec["dW_jfb_rows"] = jfb["dW"][idx].tolist()
    imp = orc.backward(p.W, C, p.tau, dist, p.G, "implicit", tol=0.0, max_iter=5, alpha=1.0)
    rec["dW_implicit5_rows"] = imp["dW"][idx].tolist()
    rec["implicit5_alpha"] = imp["alpha"]
    rec["implicit5_iters"] = imp["iters"]
    rec["oracle_seconds"] = round(time.time() - t0, 1)
    dump(rec, out)
    print(name, dist, "steps", steps, "%.0fs" % (time.time() - t0), flush=True)


def capped_layer(name, dist, out, stages=(50, 100, 150, 200), bwd_passes=(10, 50)):
    """The configs whose forward solve ends at its iteration cap: the codebook along the trajectory (every stage
    continues the previous one, which Alg. 1 does anyway: its state is the codebook alone), the result at the cap,
    and there JFB and the averaged iteration of Sec. 4.2 held to fixed pass counts (tol = 0)."""
    p = wl.make_problem(name, dist)
    assert stages[-1] == p.max_iter
    t0 = time.time()
    k, d = p.cfg.k, p.cfg.d
    idx = np.unique(np.concatenate([sample_rows(p.cfg.m, 81, 2048), np.arange(p.cfg.m - 64, p.cfg.m),
                                    np.arange(64)]))
    rec = dict(note=NOTE, config=name, dist=dist, m=p.cfg.m, d=d, k=k, tau=p.tau, tol=p.tol, max_iter=p.max_iter,
               stages=list(stages), C_at_stage=[], residual_at_stage=[], sample_rows=idx.tolist())
    C = p.C0
    done = 0
    stopped = False
    # the forward trajectory takes most of an hour at k = 256: every finished stage is kept beside the output (a file
    # git ignores), so that an interrupted run continues from its last stage instead of starting over
    ckpt = out + ".ckpt.json"
    if os.path.exists(ckpt):
        with open(ckpt) as f:
            ck = json.load(f)
        if ck["stages"] == list(stages) and ck["tau"] == p.tau and ck["m"] == p.cfg.m:
            rec["C_at_stage"], rec["residual_at_stage"] = ck["C_at_stage"], ck["residual_at_stage"]
            done = stages[len(rec["C_at_stage"]) - 1]
            C = np.array(rec["C_at_stage"][-1], dtype=np.float64)
            print(name, dist, "continuing after", done, "evaluations", flush=True)
    for s in stages:
        if s <= done:
            continue
        fw = orc.soft_kmeans(p.W, C, p.tau, p.tol, s - done, dist)
        C = fw["C"]
        done += fw["iters"]
        rec["C_at_stage"].append(C.tolist())
        rec["residual_at_stage"].append(fw["residual"])
        print(name, dist, "evaluations", done, "residual %.3e" % fw["residual"], "%.0fs" % (time.time() - t0),
              flush=True)
        if fw["converged"]:
            stopped = True
            break
        with open(ckpt, "w") as f:  # full precision: the next stage starts from these numbers
            json.dump(dict(stages=list(stages), tau=p.tau, m=p.cfg.m, C_at_stage=rec["C_at_stage"],
                           residual_at_stage=rec["residual_at_stage"]), f)
    rec.update(iters=done, converged=stopped, residual=rec["residual_at_stage"][-1], C=C.tolist())
    Wq = orc.soft_quantize(p.W, C, p.tau, dist)
    rec["Wq_rows"] = Wq[idx].tolist()
    rec["Wq_norm"] = float(np.linalg.norm(Wq))
    rec["Wq_colsum"] = Wq.sum(0).tolist()
    del Wq
    A = orc.attention(p.W, C, p.tau, dist)
    Fv, n = orc.mstep(A, p.W, C)
    del A
    rec["n"] = n.tolist()
    rec["F_at_C"] = Fv.tolist()
    jfb = orc.backward(p.W, C, p.tau, dist, p.G, "jfb")
    rec["v"] = jfb["v"].tolist()
    rec["dW_jfb_rows"] = jfb["dW"][idx].tolist()
    rec["dW_jfb_norm"] = float(np.linalg.norm(jfb["dW"]))
    rec["dW_jfb_colsum"] = jfb["dW"].sum(0).tolist()
    rec["dW_jfb_absmax"] = float(np.abs(jfb["dW"]).max())
    del jfb
    print(name, dist, "jfb done", "%.0fs" % (time.time() - t0), flush=True)
    rec["implicit"] = []
    for passes in bwd_passes:
        imp = orc.backward(p.W, C, p.tau, dist, p.G, "implicit", tol=0.0, max_iter=passes, alpha=1.0)
        rec["implicit"].append(dict(max_iter=passes, iters=imp["iters"], alpha=imp["alpha"], residual=imp["residual"],
                                    g=imp["g"].tolist(), dW_rows=imp["dW"][idx].tolist(),
                                    dW_norm=float(np.linalg.norm(imp["dW"])), dW_colsum=imp["dW"].sum(0).tolist(),
                                    dW_absmax=float(np.abs(imp["dW"]).max())))
        print(name, dist, "implicit", passes, "passes ->", imp["iters"], "alpha", imp["alpha"],
              "%.0fs" % (time.time() - t0), flush=True)
        del imp
    rec["oracle_seconds"] = round(time.time() - t0, 1)
    dump(rec, out)


def sweep(out):
    """The ResNet18 sweep (Alg. 2's loop over layers): all 21 tensors at k = 2 and k = 4, both energies."""
    recs = []
    t0 = time.time()
    for idx_t in range(len(wl.RESNET18_TENSORS)):
        for k in (2, 4):
            for dist in (wl.DIST_L2, wl.DIST_SQL2):
                cfg = wl.sweep_config(idx_t, k, dist)
                p = wl.make_problem(cfg, dist)
                fw = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, p.max_iter, dist)
                C = fw["C"]
                rows = sample_rows(cfg.m, 80 + idx_t, 48)
                dense = orc.backward(p.W, C, p.tau, dist, p.G, "dense")
                jfb = orc.backward(p.W, C, p.tau, dist, p.G, "jfb")
                it30 = orc.backward(p.W, C, p.tau, dist, p.G, "implicit", tol=0.0, max_iter=30, alpha=1.0)
                A = orc.attention(p.W, C, p.tau, dist)
                n = orc.mstep(A, p.W, C)[1]
                del A
                recs.append(dict(tensor=idx_t, k=k, dist=dist, m=cfg.m, tau=p.tau, iters=fw["iters"],
                                 converged=fw["converged"], residual=fw["residual"], C=C.tolist(), n=n.tolist(),
                                 sample_rows=rows.tolist(),
                                 Wq_rows=orc.soft_quantize(p.W[rows], C, p.tau, dist).tolist(),
                                 v=dense["v"].tolist(), g_dense=dense["g"].tolist(),
                                 dW_implicit_rows=dense["dW"][rows].tolist(), dW_jfb_rows=jfb["dW"][rows].tolist(),
                                 dW_implicit_norm=float(np.linalg.norm(dense["dW"])),
                                 dW_jfb_norm=float(np.linalg.norm(jfb["dW"])),
                                 implicit30=dict(iters=it30["iters"], alpha=it30["alpha"], g=it30["g"].tolist(),
                                                 dW_rows=it30["dW"][rows].tolist(),
                                                 dW_norm=float(np.linalg.norm(it30["dW"])))))
                print("C5", idx_t, k, dist, fw["iters"], fw["converged"], "%.0fs" % (time.time() - t0), flush=True)
    dump(dict(note=NOTE, cases=recs), out)

def main():
    which = sys.argv[1:] or ["C2", "C3", "C4", "P16", "C5", "C4cap", "P16cap"]
    for name in which:
        if name in ("C2", "C3"):
            for dist in (wl.DIST_L2, wl.DIST_SQL2):
                solved_layer(name, dist, os.path.join(HERE, f"{name}_{wl.DIST_NAMES[dist]}.json"))
        elif name in ("C4", "P16"):
            for dist in (wl.DIST_L2, wl.DIST_SQL2):
                stepwise_layer(name, dist, os.path.join(HERE, f"{name}_{wl.DIST_NAMES[dist]}.json"),
                               steps=12 if name == "C4" else 25)
        elif name == "C5":
            sweep(os.path.join(HERE, "C5_sweep.json"))
        elif name.split(":")[0] in ("C4cap", "P16cap"):
            base = name.split(":")[0][:-3]
            for dist in (wl.DIST_L2, wl.DIST_SQL2):
                if ":" in name and wl.DIST_NAMES[dist] != name.split(":")[1]:
                    continue
                capped_layer(base, dist, os.path.join(HERE, f"{base}_{wl.DIST_NAMES[dist]}_cap.json"))


if __name__ == "__main__":
    main()
