"""Full-size parity of the HIP path against stored oracle results (tests/golden/*.json).

The fixtures are written by tests/golden/make_golden.py, which calls only oracle/; the paper prints no
worked example.  The launch configuration is the one bench.py times (path AUTO).  Tolerances as in
test_gpu_parity.py: 1e-4 norm-wise on C* / Wq / F, 1e-3 on gradients.
"""
import json
import os

import numpy as np
import pytest
import torch

from oracle import idkm_oracle as orc
from paper_2312_07759_amd import binding
from paper_2312_07759_amd import workloads as wl

pytestmark = pytest.mark.gpu

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL_VAL = 1e-4
TOL_GRAD = 1e-3


def rel(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / (den if den > 0 else 1.0))


def load(name):
    path = os.path.join(GOLD, name)
    if not os.path.exists(path):
        pytest.skip(f"{name} has not been generated")
    with open(path) as f:
        return json.load(f)


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("dist", [wl.DIST_L2, wl.DIST_SQL2])
@pytest.mark.parametrize("name", ["C2", "C3"])
def test_full_size_solved_layers(ctx, name, dist):
    g = load(f"{name}_{wl.DIST_NAMES[dist]}.json")
    p = wl.make_problem(name, dist)
    W, C0, G = (torch.from_numpy(x).cuda() for x in (p.W, p.C0, p.G))
    out = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_Wq=True, want_assign=True)
    info = out["info"]
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, g["C"]) < TOL_VAL, (info, g["iters"])
    assert abs(info.iters - g["iters"]) <= 2
    idx = np.array(g["sample_rows"])
    Wq = out["Wq"].cpu().numpy()
    assert rel(Wq[idx], g["Wq_rows"]) < 10 * TOL_VAL
    # the E-step outputs at the GPU's own C*, recomputed by the oracle on the sampled rows
    assert rel(Wq[idx], orc.soft_quantize(p.W[idx], Cg, p.tau, dist)) < TOL_VAL
    assert np.array_equal(out["assign"].cpu().numpy()[idx], orc.hard_assign_f32(p.W[idx], Cg))
    # properties that hold at any size: convex combinations of the codebook; every assignment is a valid index
    assert Wq.min() >= Cg.min() - 1e-6 and Wq.max() <= Cg.max() + 1e-6
    a = out["assign"].cpu().numpy()
    assert a.min() >= 0 and a.max() < p.cfg.k

    bj = ctx.backward(G, binding.BWD_JFB)
    dj = bj["dW"].cpu().numpy()
    assert rel(dj[idx], g["dW_jfb_rows"]) < TOL_GRAD
    assert abs(np.linalg.norm(dj.astype(np.float64)) / g["dW_jfb_norm"] - 1) < TOL_GRAD
    # explicit Jacobian + direct solve: the same linear system the oracle solved by Gaussian elimination
    bd = ctx.backward(G, binding.BWD_DENSE)
    dd = bd["dW"].cpu().numpy()
    assert bd["info"].converged
    assert rel(dd[idx], g["dW_implicit_rows"]) < TOL_GRAD, rel(dd[idx], g["dW_implicit_rows"])
    assert abs(np.linalg.norm(dd.astype(np.float64)) / g["dW_implicit_norm"] - 1) < TOL_GRAD
    bi = ctx.backward(G, binding.BWD_IMPLICIT, tol=1e-7, max_iter=20000, alpha=1.0)
    di = bi["dW"].cpu().numpy()
    if bi["info"].converged:
        assert rel(di[idx], g["dW_implicit_rows"]) < TOL_GRAD, (bi["info"], rel(di[idx], g["dW_implicit_rows"]))
        assert abs(np.linalg.norm(di.astype(np.float64)) / g["dW_implicit_norm"] - 1) < TOL_GRAD
        # translation invariance of the whole layer (holds for the implicit gradient at any size)
        col = di.astype(np.float64).sum(0)
        scale = np.abs(p.G.astype(np.float64)).sum(0) / np.sqrt(p.cfg.m)
        assert np.all(np.abs(col - np.array(g["G_colsum"])) < 0.05 * scale + 1e-3 * np.abs(g["G_colsum"]))
    else:  # the plain iteration did not meet the stop rule within the cap: it must at least be finite
        assert np.isfinite(di).all()


@pytest.mark.parametrize("dist", [wl.DIST_L2, wl.DIST_SQL2])
@pytest.mark.parametrize("name", ["C4", "P16"])
def test_full_size_stepwise(ctx, name, dist):
    g = load(f"{name}_{wl.DIST_NAMES[dist]}.json")
    p = wl.make_problem(name, dist)
    W, C0, G = (torch.from_numpy(x).cuda() for x in (p.W, p.C0, p.G))
    Cp, n = ctx.step_F(W, C0, p.tau, dist)
    assert rel(Cp.cpu().numpy(), g["F_at_C0"]) < TOL_VAL
    assert rel(n.cpu().numpy(), g["n_at_C0"]) < TOL_VAL
    u = ctx.step_JCT(torch.tensor(g["g"], dtype=torch.float32).cuda()).cpu().numpy()
    assert rel(u, g["JCTg_at_C0"]) < TOL_GRAD
    out = ctx.forward(W, C0, p.tau, 0.0, g["steps"], dist, want_Wq=True)
    assert out["info"].iters == g["steps"]
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, g["C_after_steps"]) < TOL_VAL
    idx = np.array(g["sample_rows"])
    assert rel(out["Wq"].cpu().numpy()[idx], g["Wq_rows"]) < 10 * TOL_VAL
    bj = ctx.backward(G, binding.BWD_JFB)
    assert rel(bj["dW"].cpu().numpy()[idx], g["dW_jfb_rows"]) < TOL_GRAD
    bi = ctx.backward(G, binding.BWD_IMPLICIT, tol=0.0, max_iter=5, alpha=1.0)
    assert bi["info"].iters == g["implicit5_iters"] and bi["info"].alpha == g["implicit5_alpha"]
    assert rel(bi["dW"].cpu().numpy()[idx], g["dW_implicit5_rows"]) < TOL_GRAD


def test_resnet18_sweep_cross_section(ctx):
    g = load("C5_sweep.json")
    for c in g["cases"]:
        cfg = wl.sweep_config(c["tensor"], c["k"], c["dist"])
        p = wl.make_problem(cfg, c["dist"])
        W, C0, G = (torch.from_numpy(x).cuda() for x in (p.W, p.C0, p.G))
        out = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, c["dist"], want_Wq=True)
        tag = (c["tensor"], c["k"], c["dist"], out["info"], c["iters"])
        assert rel(out["C"].cpu().numpy(), c["C"]) < TOL_VAL, tag
        assert abs(out["info"].iters - c["iters"]) <= 2, tag
        idx = np.array(c["sample_rows"])
        assert rel(out["Wq"].cpu().numpy()[idx], c["Wq_rows"]) < 10 * TOL_VAL, tag
        bj = ctx.backward(G, binding.BWD_JFB)
        assert rel(bj["dW"].cpu().numpy()[idx], c["dW_jfb_rows"]) < TOL_GRAD, tag
        bi = ctx.backward(G, binding.BWD_IMPLICIT, tol=1e-7, max_iter=20000, alpha=1.0)
        if bi["info"].converged:
            assert rel(bi["dW"].cpu().numpy()[idx], c["dW_implicit_rows"]) < TOL_GRAD, tag
