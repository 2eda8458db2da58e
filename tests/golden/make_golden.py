#!/usr/bin/env python3
"""Writes the full-size expected values under tests/golden/ from the CPU oracle alone.

The paper prints no worked numeric example, so nothing here is the paper's: every stored number is
computed by oracle/idkm_oracle.py (numpy float64) on the seeded inputs of
paper_2312_07759_amd/workloads.py.  The HIP path is never imported or run.  The full-size oracle
runs take minutes (a forward solve of the 3x3x256x256 layer is ~100 s), which is why they are
stored instead of being recomputed inside the GPU tests.

  python tests/golden/make_golden.py C2 C3 C4 P16 C5      (any subset; default: all)
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


def sweep(out):
    """A cross-section of the ResNet18 sweep: small, medium and 1x1 tensors at k = 2 and k = 4."""
    recs = []
    for idx_t in (0, 1, 9, 14, 19):
        for k in (2, 4):
            for dist in (wl.DIST_L2, wl.DIST_SQL2):
                cfg = wl.sweep_config(idx_t, k, dist)
                p = wl.make_problem(cfg, dist)
                fw = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, p.max_iter, dist)
                C = fw["C"]
                rows = sample_rows(cfg.m, 80 + idx_t, 48)
                dense = orc.backward(p.W, C, p.tau, dist, p.G, "dense")
                jfb = orc.backward(p.W, C, p.tau, dist, p.G, "jfb")
                recs.append(dict(tensor=idx_t, k=k, dist=dist, m=cfg.m, tau=p.tau, iters=fw["iters"],
                                 converged=fw["converged"], C=C.tolist(), sample_rows=rows.tolist(),
                                 Wq_rows=orc.soft_quantize(p.W[rows], C, p.tau, dist).tolist(),
                                 dW_implicit_rows=dense["dW"][rows].tolist(), dW_jfb_rows=jfb["dW"][rows].tolist()))
                print("C5", idx_t, k, dist, fw["iters"], fw["converged"], flush=True)
    dump(dict(note=NOTE, cases=recs), out)


def main():
    which = sys.argv[1:] or ["C2", "C3", "C4", "P16", "C5"]
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


if __name__ == "__main__":
    main()
