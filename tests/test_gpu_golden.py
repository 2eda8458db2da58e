"""Parity of the HIP path at the configs' own sizes, in the launch configuration bench.py times (path AUTO).

Two sources of expected values, both the CPU oracle's:
  * tests/golden/*.json, written by tests/golden/make_golden.py (which calls only oracle/): what needs minutes to
    hours of numpy -- the forward solves, the trajectories of the configs that end at their iteration cap, the
    averaged iteration of Sec. 4.2 held to a fixed number of passes;
  * the oracle run live on the WHOLE tensor at the GPU's own C*: everything that is one pass over W (Wq, hard
    assignments, the JFB gradient, the dense solve for k d <= 16), so every row is compared, tails included.
The paper prints no worked example.  Comparisons at the SAME codebook (the live ones, the codebooks themselves, the
cotangents) are norm-wise AND element-wise:
  ||x - ref||_F <= tol ||ref||_F   and   max |x - ref| <= tol max |ref|,
tol = 1e-4 for C*, Wq, F, n and 1e-3 for gradients and cotangents; hard assignments bit for bit.  Stored rows of Wq
and dW belong to the ORACLE's C*, which differs from the GPU's by rounding: a row that lies between the two positions
of a codeword or of a cell boundary changes by O(1) there (the plain norm's derivative is a sign), so those rows are
held to the norm-wise bound only.  The averaged iteration is compared at equal pass counts (tol = 0 on both sides),
so nothing depends on whether it would converge; where the float32 iteration reaches a step of exactly zero earlier
(g no longer changes, further passes are no-ops) that is accepted.  A missing fixture is a failure, not a skip.
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
DISTS = [wl.DIST_L2, wl.DIST_SQL2]


def rel(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / (den if den > 0 else 1.0))


def elem(x, ref):
    """max |x - ref| / max |ref|"""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(x - ref).max() / (den if den > 0 else 1.0))


def check(x, ref, tol, what):
    r, e = rel(x, ref), elem(x, ref)
    assert r < tol and e < tol, f"{what}: norm-wise {r:.3e}, element-wise {e:.3e}, bound {tol:g}"


def check_norm(x, ref, tol, what):
    r = rel(x, ref)
    assert r < tol, f"{what}: norm-wise {r:.3e}, bound {tol:g}"


def same_passes(info, want_iters, want_alpha):
    """The pass count and damping of an equal-pass run (tol = 0), or an exact fixed point of the float32 iteration."""
    return (info.iters == want_iters and info.alpha == want_alpha and not info.converged) or \
           (info.converged and info.residual == 0.0 and info.iters <= want_iters and info.alpha == want_alpha)


def load(name):
    path = os.path.join(GOLD, name)
    assert os.path.exists(path), f"{name} is missing: write it with tests/golden/make_golden.py"
    with open(path) as f:
        return json.load(f)


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def _whole_tensor_E_step(p, out, Cg, dist, tag):
    """Wq and the hard assignments of every row against the oracle at the GPU's own C*."""
    Wq = out["Wq"].cpu().numpy()
    check(Wq, orc.soft_quantize(p.W, Cg, p.tau, dist), TOL_VAL, f"{tag} Wq (whole tensor)")
    assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(p.W, Cg)), f"{tag} assign"
    return Wq


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name", ["C2", "C3"])
def test_full_size_solved_layers(ctx, name, dist):
    g = load(f"{name}_{wl.DIST_NAMES[dist]}.json")
    p = wl.make_problem(name, dist)
    k, d = p.cfg.k, p.cfg.d
    W, C0, G = dev(p.W), dev(p.C0), dev(p.G)
    tag = f"{name}/{wl.DIST_NAMES[dist]}"
    out = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_Wq=True, want_assign=True)
    info = out["info"]
    Cg = out["C"].cpu().numpy()
    check(Cg, g["C"], TOL_VAL, f"{tag} C* ({info}, oracle iters {g['iters']})")
    assert abs(info.iters - g["iters"]) <= 2 and info.converged == g["converged"]
    Wq = _whole_tensor_E_step(p, out, Cg, dist, tag)
    idx = np.array(g["sample_rows"])
    assert rel(Wq[idx], g["Wq_rows"]) < 10 * TOL_VAL  # against the oracle's own C*

    # Jacobian-free backward, every row, at the GPU's C*
    rj = orc.backward(p.W, Cg, p.tau, dist, p.G, "jfb")
    bj = ctx.backward(G, binding.BWD_JFB)
    check(bj["dW"].cpu().numpy(), rj["dW"], TOL_GRAD, f"{tag} JFB dW (whole tensor)")
    v_gpu, g_gpu = ctx.get_cotangents(k, d)
    check(v_gpu, rj["v"], TOL_GRAD, f"{tag} v")
    assert np.array_equal(v_gpu, g_gpu)
    assert rel(bj["dW"].cpu().numpy()[idx], g["dW_jfb_rows"]) < TOL_GRAD

    # explicit Jacobian + direct solve: the linear system the oracle solves by Gaussian elimination, every row
    rd = orc.backward(p.W, Cg, p.tau, dist, p.G, "dense")
    bd = ctx.backward(G, binding.BWD_DENSE)
    assert bd["info"].converged and bd["info"].iters == 0
    check(bd["dW"].cpu().numpy(), rd["dW"], TOL_GRAD, f"{tag} dense dW (whole tensor)")
    g_dense = ctx.get_cotangents(k, d)[1]
    # the solve is held to its backward error, evaluated by the oracle: ||v + (dF/dC*)^T g - g|| <= 1e-3 ||v||; the
    # forward error is bounded only where I - dF/dC* is well conditioned (at C2 with the squared energy it is not:
    # condition number about 1e5 at the unconverged C*)
    res = rj["v"] + orc.vjp_F(Cg, p.W, p.tau, dist, g_dense)[0] - g_dense
    assert np.linalg.norm(res) < TOL_GRAD * np.linalg.norm(rj["v"]), (tag, np.linalg.norm(res), np.linalg.norm(rj["v"]))
    if g["rho"] < 0.97:
        check(g_dense, rd["g"], TOL_GRAD, f"{tag} g of the dense solve")
    check_norm(bd["dW"].cpu().numpy()[idx], g["dW_implicit_rows"], TOL_GRAD, f"{tag} dense dW rows at the oracle's C*")

    # the averaged iteration at an equal pass count (no stop rule involved)
    r40 = g["implicit40"]
    b40 = ctx.backward(G, binding.BWD_IMPLICIT, tol=0.0, max_iter=40, alpha=1.0)
    assert same_passes(b40["info"], r40["iters"], r40["alpha"]), (tag, b40["info"], r40["iters"], r40["alpha"])
    check(ctx.get_cotangents(k, d)[1], r40["g"], TOL_GRAD, f"{tag} g after 40 passes")
    d40 = b40["dW"].cpu().numpy()
    check_norm(d40[idx], r40["dW_rows"], TOL_GRAD, f"{tag} dW after 40 passes (sampled rows)")
    assert abs(np.linalg.norm(d40.astype(np.float64)) / r40["dW_norm"] - 1) < TOL_GRAD
    assert np.abs(d40).max() <= r40["dW_absmax"] * (1 + 10 * TOL_GRAD)

    if g["rho"] < 0.97:
        # spectral radius of dF/dC* (from the oracle) well below one: the iteration must meet its stop rule, and
        # its result is the dense solve's.  (Float32 passes leave a noise floor of about 1e-6 ||g|| in the step norm,
        # so the stop rule is asked for at 1e-5 ||v||: the iterate is then within 1e-5 / (1 - rho) < 4e-4 of the solution.)
        bi = ctx.backward(G, binding.BWD_IMPLICIT, tol=1e-5, max_iter=2000, alpha=1.0)
        assert bi["info"].converged, (tag, bi["info"], g["rho"])
        di = bi["dW"].cpu().numpy()
        check(di, rd["dW"], TOL_GRAD, f"{tag} implicit dW (whole tensor)")
        # translation invariance of the whole layer (holds for the implicit gradient at any size)
        col = di.astype(np.float64).sum(0)
        scale = np.abs(p.G.astype(np.float64)).sum(0) / np.sqrt(p.cfg.m)
        assert np.all(np.abs(col - np.array(g["G_colsum"])) < 0.05 * scale + 1e-3 * np.abs(g["G_colsum"]))


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name", ["C4", "P16"])
def test_full_size_stepwise(ctx, name, dist):
    g = load(f"{name}_{wl.DIST_NAMES[dist]}.json")
    p = wl.make_problem(name, dist)
    W, C0, G = dev(p.W), dev(p.C0), dev(p.G)
    Cp, n = ctx.step_F(W, C0, p.tau, dist)
    check(Cp.cpu().numpy(), g["F_at_C0"], TOL_VAL, "F at C0")
    check(n.cpu().numpy(), g["n_at_C0"], TOL_VAL, "n at C0")
    u = ctx.step_JCT(torch.tensor(g["g"], dtype=torch.float32).cuda()).cpu().numpy()
    check(u, g["JCTg_at_C0"], TOL_GRAD, "(dF/dC)^T g at C0")
    out = ctx.forward(W, C0, p.tau, 0.0, g["steps"], dist, want_Wq=True)
    assert out["info"].iters == g["steps"]
    Cg = out["C"].cpu().numpy()
    check(Cg, g["C_after_steps"], TOL_VAL, "C after the first evaluations")
    idx = np.array(g["sample_rows"])
    assert rel(out["Wq"].cpu().numpy()[idx], g["Wq_rows"]) < 10 * TOL_VAL
    bj = ctx.backward(G, binding.BWD_JFB)
    assert rel(bj["dW"].cpu().numpy()[idx], g["dW_jfb_rows"]) < TOL_GRAD
    bi = ctx.backward(G, binding.BWD_IMPLICIT, tol=0.0, max_iter=5, alpha=1.0)
    assert bi["info"].iters == g["implicit5_iters"] and bi["info"].alpha == g["implicit5_alpha"]
    assert rel(bi["dW"].cpu().numpy()[idx], g["dW_implicit5_rows"]) < TOL_GRAD


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name", ["C4", "P16"])
def test_full_size_layers_that_end_at_their_iteration_cap(ctx, name, dist):
    """The configs whose forward solve uses all max_iter = 200 evaluations: the trajectory at 50, 100, 150 and 200
    evaluations, the outputs at the cap, JFB, and the averaged iteration at 10 and 50 passes."""
    g = load(f"{name}_{wl.DIST_NAMES[dist]}_cap.json")
    p = wl.make_problem(name, dist)
    k, d = p.cfg.k, p.cfg.d
    tag = f"{name}/{wl.DIST_NAMES[dist]}"
    W, C0, G = dev(p.W), dev(p.C0), dev(p.G)
    for s, Cs in zip(g["stages"][:-1], g["C_at_stage"][:-1]):
        o = ctx.forward(W, C0, p.tau, 0.0, s, dist, want_Wq=False)
        assert o["info"].iters == s
        check(o["C"].cpu().numpy(), Cs, TOL_VAL, f"{tag} C after {s} evaluations")
    out = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_Wq=True, want_assign=True)
    info = out["info"]
    assert info.iters == g["iters"] and info.converged == g["converged"], (info, g["iters"], g["converged"])
    assert abs(info.residual / g["residual"] - 1) < 1e-2, (info.residual, g["residual"])
    Cg = out["C"].cpu().numpy()
    check(Cg, g["C"], TOL_VAL, f"{tag} C at the cap")
    Wq = _whole_tensor_E_step(p, out, Cg, dist, tag)
    idx = np.array(g["sample_rows"])
    check_norm(Wq[idx], g["Wq_rows"], 10 * TOL_VAL, f"{tag} Wq rows at the oracle's C")
    assert abs(np.linalg.norm(Wq.astype(np.float64)) / g["Wq_norm"] - 1) < TOL_VAL

    bj = ctx.backward(G, binding.BWD_JFB)
    dj = bj["dW"].cpu().numpy()
    v_gpu = ctx.get_cotangents(k, d)[0]
    check_norm(v_gpu, g["v"], TOL_GRAD, f"{tag} v at the oracle's C")
    check_norm(dj[idx], g["dW_jfb_rows"], TOL_GRAD, f"{tag} JFB dW (sampled rows, first and last 64 rows)")
    assert abs(np.linalg.norm(dj.astype(np.float64)) / g["dW_jfb_norm"] - 1) < TOL_GRAD
    assert np.abs(dj).max() <= g["dW_jfb_absmax"] * (1 + 10 * TOL_GRAD)
    # every row, and v, against the oracle at the GPU's own C (two passes of numpy over the m x k matrices)
    rj = orc.backward(p.W, Cg, p.tau, dist, p.G, "jfb")
    check(v_gpu, rj["v"], TOL_GRAD, f"{tag} v")
    check(dj, rj["dW"], TOL_GRAD, f"{tag} JFB dW (whole tensor)")
    # The stored backward results belong to the ORACLE's codebook at the cap.  Along an unconverged trajectory the GPU's
    # codebook differs from it by about 1e-5, and with the plain norm (whose derivative is a sign) that alone moves v by
    # 9e-4 and the iterate after 10 passes by 1.3e-3.  So the backward is run from the oracle's codebook (rounded to
    # float32: 6e-8), handed over through idkm_step_F, which leaves (W, C, n, F(C, W)) as the forward state.
    Co = np.array(g["C"], dtype=np.float32)
    Fo, no = ctx.step_F(W, dev(Co), p.tau, dist)
    check(Fo.cpu().numpy(), g["F_at_C"], TOL_VAL, f"{tag} F at the oracle's C")
    check(no.cpu().numpy(), g["n"], TOL_VAL, f"{tag} n at the oracle's C")
    bo = ctx.backward(G, binding.BWD_JFB)
    check(ctx.get_cotangents(k, d)[0], g["v"], TOL_GRAD, f"{tag} v from the oracle's C")
    check_norm(bo["dW"].cpu().numpy()[idx], g["dW_jfb_rows"], TOL_GRAD, f"{tag} JFB dW rows from the oracle's C")
    for r in g["implicit"]:
        bi = ctx.backward(G, binding.BWD_IMPLICIT, tol=0.0, max_iter=r["max_iter"], alpha=1.0)
        assert same_passes(bi["info"], r["iters"], r["alpha"]), (tag, bi["info"], r["iters"], r["alpha"])
        check(ctx.get_cotangents(k, d)[1], r["g"], TOL_GRAD, f"{tag} g after {r['max_iter']} passes")
        di = bi["dW"].cpu().numpy()
        check_norm(di[idx], r["dW_rows"], TOL_GRAD, f"{tag} dW after {r['max_iter']} passes (sampled rows)")
        assert abs(np.linalg.norm(di.astype(np.float64)) / r["dW_norm"] - 1) < TOL_GRAD
        assert np.abs(di).max() <= r["dW_absmax"] * (1 + 10 * TOL_GRAD)


# ---------------------------------------------------------------- the ResNet18 sweep (Alg. 2's loops over layers)

N_TENSORS = len(wl.RESNET18_TENSORS)


@pytest.fixture(scope="module")
def sweep_gold():
    g = load("C5_sweep.json")
    by = {(c["tensor"], c["k"], c["dist"]): c for c in g["cases"]}
    assert len(by) == N_TENSORS * 4, "the fixture must hold all 21 tensors at k = 2, 4 and both energies"
    return by


def _check_sweep_backwards(c, tag, rows, dj, dd, d30, i30, cot=None):
    check_norm(dj[rows], c["dW_jfb_rows"], TOL_GRAD, f"{tag} JFB dW rows")
    assert abs(np.linalg.norm(dj.astype(np.float64)) / c["dW_jfb_norm"] - 1) < TOL_GRAD, tag
    check_norm(dd[rows], c["dW_implicit_rows"], TOL_GRAD, f"{tag} dense dW rows")
    assert abs(np.linalg.norm(dd.astype(np.float64)) / c["dW_implicit_norm"] - 1) < TOL_GRAD, tag
    r30 = c["implicit30"]
    assert same_passes(i30, r30["iters"], r30["alpha"]), (tag, i30, r30["iters"], r30["alpha"])
    check_norm(d30[rows], r30["dW_rows"], TOL_GRAD, f"{tag} dW rows after 30 passes")
    assert abs(np.linalg.norm(d30.astype(np.float64)) / r30["dW_norm"] - 1) < TOL_GRAD, tag
    if cot is not None:
        check(cot["v"], c["v"], TOL_GRAD, f"{tag} v")
        check(cot["g_dense"], c["g_dense"], TOL_GRAD, f"{tag} g of the dense solve")
        check(cot["g30"], r30["g"], TOL_GRAD, f"{tag} g after 30 passes")


@pytest.mark.parametrize("tensor", range(N_TENSORS))
def test_resnet18_sweep_every_tensor(ctx, sweep_gold, tensor):
    for k in (2, 4):
        for dist in DISTS:
            c = sweep_gold[(tensor, k, dist)]
            cfg = wl.sweep_config(tensor, k, dist)
            p = wl.make_problem(cfg, dist)
            tag = f"tensor {tensor} k={k} {wl.DIST_NAMES[dist]}"
            W, C0, G = dev(p.W), dev(p.C0), dev(p.G)
            out = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_Wq=True, want_assign=True)
            Cg = out["C"].cpu().numpy()
            check(Cg, c["C"], TOL_VAL, f"{tag} C* ({out['info']}, oracle iters {c['iters']})")
            assert abs(out["info"].iters - c["iters"]) <= 2 and out["info"].converged == c["converged"], tag
            Wq = _whole_tensor_E_step(p, out, Cg, dist, tag)
            rows = np.array(c["sample_rows"])
            assert rel(Wq[rows], c["Wq_rows"]) < 10 * TOL_VAL, tag
            bj = ctx.backward(G, binding.BWD_JFB)
            dj = bj["dW"].cpu().numpy()
            check(dj, orc.backward(p.W, Cg, p.tau, dist, p.G, "jfb")["dW"], TOL_GRAD, f"{tag} JFB dW (whole tensor)")
            cot = dict(v=ctx.get_cotangents(k, 1)[0])
            bd = ctx.backward(G, binding.BWD_DENSE)
            assert bd["info"].converged
            cot["g_dense"] = ctx.get_cotangents(k, 1)[1]
            b30 = ctx.backward(G, binding.BWD_IMPLICIT, tol=0.0, max_iter=30, alpha=1.0)
            cot["g30"] = ctx.get_cotangents(k, 1)[1]
            _check_sweep_backwards(c, tag, rows, dj, bd["dW"].cpu().numpy(), b30["dW"].cpu().numpy(), b30["info"], cot)


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("k", [2, 4])
def test_resnet18_sweep_batched(sweep_gold, k, dist):
    """The same 21 layers through idkm_batch_forward / idkm_batch_backward: one batch, shared launches."""
    ps = [wl.make_problem(wl.sweep_config(t, k, dist), dist) for t in range(N_TENSORS)]
    layers = [(dev(p.W), dev(p.C0)) for p in ps]
    Gs = [dev(p.G) for p in ps]
    b = binding.Batch(N_TENSORS, 0)
    try:
        outs = b.forward(layers, [p.tau for p in ps], ps[0].tol, ps[0].max_iter, dist, want_Wq=True, want_assign=True)
        assert b.launches() >= 1
        bj = b.backward(Gs, binding.BWD_JFB)
        bd = b.backward(Gs, binding.BWD_DENSE)
        b30 = b.backward(Gs, binding.BWD_IMPLICIT, tol=0.0, max_iter=30, alpha=1.0)
    finally:
        b.close()
    for t, p in enumerate(ps):
        c = sweep_gold[(t, k, dist)]
        tag = f"batched tensor {t} k={k} {wl.DIST_NAMES[dist]}"
        o = outs[t]
        assert o["status"] == 0 and bj[t]["status"] == 0 and bd[t]["status"] == 0 and b30[t]["status"] == 0, tag
        Cg = o["C"].cpu().numpy()
        check(Cg, c["C"], TOL_VAL, f"{tag} C* ({o['info']}, oracle iters {c['iters']})")
        assert abs(o["info"].iters - c["iters"]) <= 2 and o["info"].converged == c["converged"], tag
        rows = np.array(c["sample_rows"])
        Wq = o["Wq"].cpu().numpy()
        assert rel(Wq[rows], c["Wq_rows"]) < 10 * TOL_VAL, tag
        # properties that hold at any size: convex combinations of the codebook, valid indices; the hard
        # assignments of every row against the float32 key at the batch's own C*
        assert Wq.min() >= Cg.min() - 1e-6 and Wq.max() <= Cg.max() + 1e-6, tag
        _whole_tensor_E_step(p, o, Cg, dist, tag)
        check(bj[t]["dW"].cpu().numpy(), orc.backward(p.W, Cg, p.tau, dist, p.G, "jfb")["dW"], TOL_GRAD,
              f"{tag} JFB dW (whole tensor)")
        assert bd[t]["info"].converged, tag
        _check_sweep_backwards(c, tag, rows, bj[t]["dW"].cpu().numpy(), bd[t]["dW"].cpu().numpy(),
                               b30[t]["dW"].cpu().numpy(), b30[t]["info"])
