"""GPU-vs-oracle parity of the HIP path, element by element, through the C ABI.

Tolerances (norm-wise relative, ||x_gpu - x_ref||_F / ||x_ref||_F):
  C*, Wq, A, one evaluation of F ........ 1e-4
  gradients, one (dF/dC)^T pass ......... 1e-3
  hard assignments ...................... bit-exact against the float32 key evaluated on the GPU's own C*
The kernels compute in float32 (float64 only in the O(k d) reductions); the oracle in float64.
"""
import numpy as np
import pytest
import torch

from oracle import idkm_oracle as orc
from paper_2312_07759_amd import binding
from paper_2312_07759_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL_VAL = 1e-4
TOL_GRAD = 1e-3
DISTS = [wl.DIST_L2, wl.DIST_SQL2]


def rel(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / (den if den > 0 else 1.0))


def dev(x, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(x), dtype=dtype).cuda()


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


# (name, m, d, k, tau relative to the data scale): spans both kernel families, ragged tails, several tiles
STEP_CASES = [
    ("k4d1", 70_001, 1, 4, 0.05),
    ("k2d1", 5_000, 1, 2, 0.1),
    ("k16d1", 33_333, 1, 16, 0.01),
    ("k8d2", 20_011, 2, 8, 0.1),
    ("k16d4", 9_999, 4, 16, 0.3),
    ("k4d2", 257, 2, 4, 0.2),
    ("k256d4", 6_007, 4, 256, 0.5),
    ("k64d1", 4_100, 1, 64, 0.02),
    ("k100d2", 3_001, 2, 100, 0.2),   # not a multiple of 64: padded lanes
    ("k3d1", 1_000, 1, 3, 0.1),       # odd k goes to the lane<->codeword family
    ("k32d8", 2_050, 8, 32, 1.0),
    ("k1d4", 300, 4, 1, 0.5),
    ("k1024d4", 2_100, 4, 1024, 0.5),  # the largest codebook the library accepts (k d = 4096)
    ("k512d8", 1_100, 8, 512, 1.0),    # the largest d
]


def _case(m, d, k, seed):
    W, C0, G = wl.random_problem(m, d, k, seed=seed, std=0.5, spread=1.5)
    return W.astype(np.float32), C0.astype(np.float32), G.astype(np.float32)


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name,m,d,k,tau", STEP_CASES, ids=[c[0] for c in STEP_CASES])
def test_one_evaluation_of_F_and_one_JCT_pass(ctx, name, m, d, k, tau, dist):
    W, C0, _ = _case(m, d, k, seed=100 + [c[0] for c in STEP_CASES].index(name))
    # move the codebook off the data rows (the plain norm is not differentiable at w == c)
    C0 = (C0 + 0.01 * np.random.default_rng(1).standard_normal(C0.shape)).astype(np.float32)
    Wd, Cd = dev(W), dev(C0)
    Cp, n = ctx.step_F(Wd, Cd, tau, dist)
    ref = orc.F(C0, W, tau, dist)
    nref = orc.mstep(orc.attention(W, C0, tau, dist), W, C0)[1]
    assert rel(Cp.cpu().numpy(), ref) < TOL_VAL
    assert rel(n.cpu().numpy(), nref) < TOL_VAL
    g = np.random.default_rng(2).standard_normal((k, d)).astype(np.float32)
    u = ctx.step_JCT(dev(g)).cpu().numpy()
    uref = orc.vjp_F(C0, W, tau, dist, g)[0]
    assert rel(u, uref) < TOL_GRAD, (name, rel(u, uref))


@pytest.mark.parametrize("path", ["stream", "persistent"])
@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("m,d,k", [(5_003, 1, 4), (4_001, 2, 8), (3_000, 4, 256), (2_000, 1, 64), (9_001, 1, 16),
                                   (3_001, 1, 2), (1_300_007, 1, 4)])
def test_rows_whose_softmax_underflows_without_a_shift(ctx, m, d, k, dist, path):
    # A few vectors sit so far from every codeword that exp(-e/tau) underflows in float32 for the whole row;
    # the forward loop must then fall back to the shifted softmax for those rows.
    W, C0, _ = _case(m, d, k, seed=500 + k)
    W[::997] += 40.0
    W[5] -= 75.0
    tau = 0.05
    ctx.set_path(binding.PATH_STREAM if path == "stream" else binding.PATH_PERSISTENT)
    try:
        out = ctx.forward(dev(W), dev(C0), tau, 0.0, 3, dist)
    finally:
        ctx.set_path(binding.PATH_AUTO)
    ref = orc.soft_kmeans(W, C0, tau, 0.0, 3, dist)
    assert out["info"].iters == 3
    assert torch.isfinite(out["C"]).all()
    assert rel(out["C"].cpu().numpy(), ref["C"]) < TOL_VAL


FWD_CASES = [
    # name, config, m (None = full size)
    ("C1", "C1", None),
    ("C2@40k", "C2", 40_013),
    ("C3@100k", "C3", 100_003),
    ("C4@6k", "C4", 6_001),
]


@pytest.mark.parametrize("path", ["stream", "persistent"])
@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name,cfg,m", FWD_CASES, ids=[c[0] for c in FWD_CASES])
def test_forward_solve_and_backward_on_config_shaped_inputs(ctx, name, cfg, m, dist, path):
    ctx.set_path(binding.PATH_STREAM if path == "stream" else binding.PATH_PERSISTENT)
    try:
        _forward_backward_case(ctx, cfg, m, dist, binding.PATH_STREAM if path == "stream" else binding.PATH_PERSISTENT)
    finally:
        ctx.set_path(binding.PATH_AUTO)


def _forward_backward_case(ctx, cfg, m, dist, expect_path):
    p = wl.make_problem(cfg, dist, m=m)
    Wd, C0d = dev(p.W), dev(p.C0)
    out = ctx.forward(Wd, C0d, p.tau, p.tol, p.max_iter, dist, want_A=True, want_Wq=True, want_assign=True)
    info = out["info"]
    assert info.path == expect_path
    ref = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, p.max_iter, dist)
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, ref["C"]) < TOL_VAL, (info, ref["iters"], rel(Cg, ref["C"]))
    # the stop decision may fall one evaluation earlier or later when the residual grazes tol
    assert abs(info.iters - ref["iters"]) <= 2, (info, ref["iters"])
    assert info.converged == ref["converged"] or abs(info.residual - p.tol) < 0.2 * p.tol
    # same evaluation count, no stop-time jitter
    ref_same = orc.soft_kmeans(p.W, p.C0, p.tau, 0.0, info.iters, dist)
    assert rel(Cg, ref_same["C"]) < TOL_VAL
    # E-step outputs against the oracle evaluated at the GPU's own C*
    assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(p.W, Cg, p.tau, dist)) < TOL_VAL
    Aref = orc.attention(p.W, Cg, p.tau, dist)
    Ag = out["A"].cpu().numpy()
    assert rel(Ag, Aref) < TOL_VAL
    np.testing.assert_allclose(Ag.sum(1), 1.0, atol=1e-5)
    assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(p.W, Cg))
    # against the oracle's own C*
    assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(p.W, ref["C"], p.tau, dist)) < 10 * TOL_VAL

    # backward at the GPU's C* (isolates the backward from forward differences)
    if p.G is not None:
        G = p.G
    else:
        G = (2.0 * (orc.soft_quantize(p.W, Cg, p.tau, dist) - p.T)).astype(np.float32)
    Gd = dev(G)
    bj = ctx.backward(Gd, binding.BWD_JFB)
    rj = orc.backward(p.W, Cg, p.tau, dist, G, "jfb")
    assert rel(bj["dW"].cpu().numpy(), rj["dW"]) < TOL_GRAD
    assert bj["info"].iters == 0 and bj["info"].path == expect_path

    kd = p.cfg.k * p.cfg.d
    passes = 60 if kd <= 64 else 25
    bi = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=passes, alpha=1.0)
    ri = orc.backward(p.W, Cg, p.tau, dist, G, "implicit", tol=0.0, max_iter=passes, alpha=1.0)
    # same pass count and same damping decisions (a divergent undamped iteration restarts with alpha/2)
    assert bi["info"].iters == ri["iters"] and not bi["info"].converged
    assert bi["info"].alpha == ri["alpha"]
    assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD, rel(bi["dW"].cpu().numpy(), ri["dW"])
    if kd <= 16 and p.cfg.k in (2, 4, 8, 16):
        # explicit Jacobian + direct solve on the GPU against the oracle's Gaussian elimination
        bd = ctx.backward(Gd, binding.BWD_DENSE)
        rd = orc.backward(p.W, Cg, p.tau, dist, G, "dense")
        assert bd["info"].converged and bd["info"].iters == 0
        assert rel(bd["dW"].cpu().numpy(), rd["dW"]) < TOL_GRAD, rel(bd["dW"].cpu().numpy(), rd["dW"])
    if kd <= 64:
        # Run to the stop rule and compare with the dense solve of the same linear system.  Whether the undamped
        # iteration can meet its stop rule is decided by the oracle: the spectral radius of dF/dC* at this C*.  (The
        # equal-pass comparison above holds either way.)
        rho = float(np.abs(np.linalg.eigvals(orc.jacobian_C(Cg, p.W, p.tau, dist))).max())
        if rho < 0.97:
            # (float32 passes leave a noise floor of about 1e-6 ||g|| in the step norm, so the stop rule is asked for
            # at 1e-5 ||v||; with rho < 0.97 the iterate is then within 1e-5 / (1 - rho) < 4e-4 of the solution)
            bc = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=1e-5, max_iter=5000, alpha=1.0)
            assert bc["info"].converged, (bc["info"], rho)
            rd = orc.backward(p.W, Cg, p.tau, dist, G, "dense")
            assert rel(bc["dW"].cpu().numpy(), rd["dW"]) < TOL_GRAD
            # translation invariance of the layer: the implicit gradient sums to the upstream sum
            np.testing.assert_allclose(bc["dW"].double().sum(0).cpu().numpy(), G.astype(np.float64).sum(0),
                                       rtol=2e-3, atol=2e-3 * np.abs(G).sum() / len(G) ** 0.5)


@pytest.mark.parametrize("dist", DISTS)
def test_damped_solve_agrees_with_the_undamped_one(ctx, dist):
    p = wl.make_problem("C1", dist)
    out = ctx.forward(dev(p.W), dev(p.C0), p.tau, p.tol, p.max_iter, dist)
    Cg = out["C"].cpu().numpy()
    G = (2.0 * (orc.soft_quantize(p.W, Cg, p.tau, dist) - p.T)).astype(np.float32)
    Gd = dev(G)
    a = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=1e-7, max_iter=20000, alpha=1.0)
    b = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=1e-7, max_iter=20000, alpha=0.25)
    assert a["info"].converged and b["info"].converged
    assert b["info"].iters > a["info"].iters and b["info"].alpha == 0.25
    assert rel(b["dW"].cpu().numpy(), a["dW"].cpu().numpy()) < 1e-4
    rd = orc.backward(p.W, Cg, p.tau, dist, G, "dense")
    assert rel(a["dW"].cpu().numpy(), rd["dW"]) < TOL_GRAD
    ro = orc.backward(p.W, Cg, p.tau, dist, G, "implicit", tol=1e-7, max_iter=20000, alpha=0.25)
    # slow linear convergence: float32 rounding in the passes may move the stop by a few passes
    assert abs(ro["iters"] - b["info"].iters) <= 2 + 0.02 * ro["iters"]


@pytest.mark.parametrize("setting", ["0", "2"])
@pytest.mark.parametrize("cfg,m", [("C3", 300_007), ("C3", 70_001), ("C2", 100_003), ("P16", 80_011), ("C3", 8_003), ("C2", 21_001)],
                         ids=["C3@300k", "C3@70k", "C2@100k", "P16@80k", "C3@8k", "C2@21k"])
def test_forms_of_the_grid_exchange_agree(ctx, cfg, m, setting, monkeypatch):
    """Teams of 8 or more workgroups exchange their sums in two levels (inside a die through its L2, then across dies).
    IDKM_TREE=0 (read when a context is created) keeps the one-level exchange; IDKM_TREE=2 takes the two levels with
    every store at device scope, the form a workgroup falls back to when it does not run on its leader's die.  Same
    sums in a different order: the solves agree to rounding, and each form is held to the oracle."""
    dist = wl.DIST_SQL2
    p = wl.make_problem(cfg, dist, m=m)      # 256, 69, 98, 79, 8 and 21 workgroups: full and partly filled dies
    Wd, C0d, Gd = dev(p.W), dev(p.C0), dev(p.G)
    monkeypatch.setenv("IDKM_TREE", setting)
    other = binding.Context(0)
    monkeypatch.delenv("IDKM_TREE")
    try:
        res = []
        for c in (ctx, other):
            o = c.forward(Wd, C0d, p.tau, p.tol, p.max_iter, dist)
            b = c.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=25)
            assert o["info"].path == binding.PATH_PERSISTENT and b["info"].iters == 25
            res.append((o["C"].cpu().numpy(), o["Wq"].cpu().numpy(), o["info"].iters, b["dW"].cpu().numpy()))
    finally:
        other.close()
    assert abs(res[0][2] - res[1][2]) <= 1
    assert rel(res[1][0], res[0][0]) < 1e-5 and rel(res[1][1], res[0][1]) < 1e-5 and rel(res[1][3], res[0][3]) < 1e-4
    ref = orc.soft_kmeans(p.W, p.C0, p.tau, 0.0, res[1][2], dist)
    assert rel(res[1][0], ref["C"]) < TOL_VAL
    ri = orc.backward(p.W, res[1][0], p.tau, dist, p.G, "implicit", tol=0.0, max_iter=25)
    assert rel(res[1][3], ri["dW"]) < TOL_GRAD


def test_results_are_bitwise_reproducible(ctx):
    p = wl.make_problem("C3", wl.DIST_SQL2, m=200_001)
    Wd, C0d, Gd = dev(p.W), dev(p.C0), dev(p.G)
    runs = []
    for _ in range(2):
        o = ctx.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        b = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=1e-6, max_iter=300)
        runs.append((o["C"].cpu(), o["Wq"].cpu(), o["info"].iters, b["dW"].cpu(), b["info"].iters))
    assert runs[0][2] == runs[1][2] and runs[0][4] == runs[1][4]
    for x, y in zip(runs[0], runs[1]):
        if isinstance(x, torch.Tensor):
            assert torch.equal(x, y)


DENSE_CASES = [("k2d1", 3_001, 1, 2), ("k4d1", 70_001, 1, 4), ("k8d1", 9_000, 1, 8), ("k2d2", 4_097, 2, 2),
               ("k4d2", 5_000, 2, 4), ("k8d2", 6_001, 2, 8), ("k2d4", 2_500, 4, 2), ("k4d4", 7_003, 4, 4)]


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name,m,d,k", DENSE_CASES, ids=[c[0] for c in DENSE_CASES])
def test_dense_backward_matches_the_gaussian_solve(ctx, name, m, d, k, dist):
    W, C0, G = _case(m, d, k, seed=300 + [c[0] for c in DENSE_CASES].index(name))
    tau = 0.3
    out = ctx.forward(dev(W), dev(C0), tau, 1e-6, 300, dist)
    Cg = out["C"].cpu().numpy()
    rd = orc.backward(W, Cg, tau, dist, G, "dense")
    kd = k * d
    one_launch = kd * kd + kd * d + kd <= 32      # the sums fit one exchange line: k=2 (d=1,2) and k=4 (d=1)
    for path in (binding.PATH_STREAM, binding.PATH_PERSISTENT, binding.PATH_AUTO):
        ctx.set_path(path)
        try:
            bd = ctx.backward(dev(G), binding.BWD_DENSE)
        finally:
            ctx.set_path(binding.PATH_AUTO)
        assert bd["info"].converged and bd["info"].iters == 0
        want = binding.PATH_STREAM if (path == binding.PATH_STREAM or not one_launch) else binding.PATH_PERSISTENT
        assert bd["info"].path == want
        assert rel(bd["dW"].cpu().numpy(), rd["dW"]) < TOL_GRAD, (path, rel(bd["dW"].cpu().numpy(), rd["dW"]))


def test_dense_backward_is_refused_beyond_its_size_limit(ctx):
    W, C0, G = _case(2_000, 2, 16, seed=400)  # k d = 32 > 16
    ctx.forward(dev(W), dev(C0), 0.3, 1e-6, 5, wl.DIST_SQL2)
    with pytest.raises(binding.IdkmError) as e:
        ctx.backward(dev(G), binding.BWD_DENSE)
    assert e.value.status == 6
    W, C0, G = _case(2_000, 1, 64, seed=401)  # lane<->codeword family
    ctx.forward(dev(W), dev(C0), 0.3, 1e-6, 5, wl.DIST_SQL2)
    with pytest.raises(binding.IdkmError) as e:
        ctx.backward(dev(G), binding.BWD_DENSE)
    assert e.value.status == 6


def test_edge_cases(ctx):
    d = wl.DIST_SQL2
    # m == k == 1
    W = dev(np.array([[0.25]], dtype=np.float32))
    o = ctx.forward(W, dev(np.array([[1.0]], dtype=np.float32)), 0.1, 1e-6, 10, d, want_assign=True)
    assert abs(o["C"].item() - 0.25) < 1e-7 and o["info"].converged and o["assign"].item() == 0
    # max_iter = 1 and tol = 0: exactly one evaluation, reported as not converged
    p = wl.make_problem("C1", d)
    o = ctx.forward(dev(p.W), dev(p.C0), p.tau, 0.0, 1, d)
    assert o["info"].iters == 1 and not o["info"].converged
    assert rel(o["C"].cpu().numpy(), orc.F(p.C0, p.W, p.tau, d)) < TOL_VAL
    # a codeword far from all data underflows to zero mass in float32: it keeps its centre, and is counted
    C0 = p.C0.copy()
    C0[3, 0] = 50.0
    o = ctx.forward(dev(p.W), dev(C0), p.tau, p.tol, 5, d)
    assert o["info"].empty_clusters == 1 and o["C"][3, 0].item() == 50.0
    b = ctx.backward(dev(np.ones_like(p.W)), binding.BWD_JFB)
    assert torch.isfinite(b["dW"]).all()
    # k == m
    W4 = np.array([[0.0], [1.0], [2.0], [3.5]], dtype=np.float32)
    o = ctx.forward(dev(W4), dev(W4.copy()), 0.01, 1e-6, 10, d, want_assign=True)
    assert o["assign"].cpu().tolist() == [0, 1, 2, 3]
    np.testing.assert_allclose(o["C"].cpu().numpy(), W4, atol=1e-6)


def test_an_expired_device_wait_is_reported_and_the_context_stays_usable(ctx):
    # The host forces the condition: with a spin limit of 0 the first unsuccessful poll of a grid-wide wait gives
    # up, every workgroup leaves the kernel normally, and the call reports a device error.
    p = wl.make_problem("C3", wl.DIST_SQL2, m=100_003)
    Wd, C0d = dev(p.W), dev(p.C0)
    ctx.set_path(binding.PATH_PERSISTENT)
    try:
        ctx.set_spin_limit(0)
        with pytest.raises(binding.IdkmError) as e:
            ctx.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        assert e.value.status == 3
        with pytest.raises(binding.IdkmError) as e:  # no forward state was left behind
            ctx.backward(dev(p.G), binding.BWD_JFB)
        assert e.value.status == 5
        ctx.set_spin_limit(1 << 20)
        out = ctx.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        ref = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        assert rel(out["C"].cpu().numpy(), ref["C"]) < TOL_VAL
    finally:
        ctx.set_spin_limit(1 << 20)
        ctx.set_path(binding.PATH_AUTO)


@pytest.mark.parametrize("kind", ["one call", "batched"])
def test_an_expired_wait_is_answered_by_the_stream_path_under_auto(ctx, kind):
    """A persistent solve that cannot run to its end (here: every device-side wait gives up at its first unsuccessful
    poll; all kernels still exit normally) is solved again on the stream path when the path is AUTO."""
    p = wl.make_problem("C3", wl.DIST_SQL2, m=300_007)   # 256 workgroups: the exchange has somebody to wait for
    Wd, C0d, Gd = dev(p.W), dev(p.C0), dev(p.G)
    ref = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
    if kind == "one call":
        ctx.set_spin_limit(0)
        try:
            out = ctx.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
            bj = ctx.backward(Gd, binding.BWD_JFB)
            bi = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=20)
        finally:
            ctx.set_spin_limit(1 << 20)
    else:
        b = binding.Batch(2, 0)
        try:
            for i in range(2):
                b.context_set_spin_limit(i, 0)
            o2 = b.forward([(Wd, C0d), (Wd, C0d)], p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
            j2 = b.backward([Gd, Gd], binding.BWD_JFB)
            i2 = b.backward([Gd, Gd], binding.BWD_IMPLICIT, tol=0.0, max_iter=20)
            assert all(x["status"] == 0 for x in o2 + j2 + i2)
            out, bj, bi = o2[1], j2[1], i2[1]
        finally:
            b.close()
    assert out["info"].path == binding.PATH_STREAM and bj["info"].path == binding.PATH_STREAM
    assert bi["info"].path == binding.PATH_STREAM and bi["info"].iters == 20
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, ref["C"]) < TOL_VAL
    assert rel(bj["dW"].cpu().numpy(), orc.backward(p.W, Cg, p.tau, wl.DIST_SQL2, p.G, "jfb")["dW"]) < TOL_GRAD
    ri = orc.backward(p.W, Cg, p.tau, wl.DIST_SQL2, p.G, "implicit", tol=0.0, max_iter=20)
    assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD


@pytest.mark.parametrize("path", ["stream", "persistent"])
def test_a_cotangent_that_overflows_is_reported_as_non_finite(ctx, path):
    """Upstream gradients so large that float32 overflows somewhere in the backward (in v, or only in the (dF/dC)^T
    passes, for every damping factor the restart rule tries): the call must say so -- IDKM_ERR_NONFINITE -- and never
    return IDKM_OK with a gradient that holds NaN or Inf."""
    W, C0, _ = _case(20_011, 1, 4, seed=77)
    ctx.set_path(binding.PATH_STREAM if path == "stream" else binding.PATH_PERSISTENT)
    refused = 0
    try:
        ctx.forward(dev(W), dev(C0), 0.002, 1e-6, 50, wl.DIST_SQL2)
        for scale in (1e28, 1e30, 1e32, 1e33, 1e34, 1e35, 1e36, 1e37):
            G = (np.random.default_rng(5).standard_normal(W.shape) * scale).astype(np.float32)
            try:
                r = ctx.backward(dev(G), binding.BWD_IMPLICIT, tol=1e-6, max_iter=50, alpha=1.0)
                assert torch.isfinite(r["dW"]).all(), (scale, r["info"])
            except binding.IdkmError as e:
                assert e.status == 4, (scale, e)
                refused += 1
    finally:
        ctx.set_path(binding.PATH_AUTO)
    assert refused >= 1


def test_cotangents_and_kernel_timing_accessors(ctx):
    p = wl.make_problem("C1", wl.DIST_SQL2)
    Wd, C0d = dev(p.W), dev(p.C0)
    fresh = binding.Context(0)
    try:
        fresh.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        with pytest.raises(binding.IdkmError) as e:      # no backward since this forward
            fresh.get_cotangents(4, 1)
        assert e.value.status == 5
        with pytest.raises(binding.IdkmError) as e:      # timing is off
            fresh.last_kernel_ms()
        assert e.value.status == 1
        fresh.set_kernel_timing(True)
        fresh.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        t = fresh.last_kernel_ms()
        assert 0.0 < t < 50.0
        fresh.set_path(binding.PATH_STREAM)
        fresh.forward(Wd, C0d, p.tau, p.tol, p.max_iter, wl.DIST_SQL2)
        with pytest.raises(binding.IdkmError):            # the stream path is many launches: nothing to report
            fresh.last_kernel_ms()
        G = dev(np.ones_like(p.W))
        fresh.backward(G, binding.BWD_JFB)
        v, g = fresh.get_cotangents(4, 1)
        assert np.array_equal(v, g) and np.isfinite(v).all() and np.abs(v).max() > 0
    finally:
        fresh.close()


def test_error_paths(ctx):
    d = wl.DIST_SQL2
    W = dev(np.zeros((8, 1), dtype=np.float32))
    C0 = dev(np.zeros((2, 1), dtype=np.float32))
    fresh = binding.Context(0)
    with pytest.raises(binding.IdkmError) as e:
        fresh.backward(W, binding.BWD_JFB)
    assert e.value.status == 5
    fresh.close()
    for kwargs, status in [
        (dict(tau=0.0), 1), (dict(tau=float("nan")), 1), (dict(tol=-1.0), 1), (dict(max_iter=0), 1), (dict(dist=7), 1),
    ]:
        args = dict(tau=0.1, tol=1e-6, max_iter=5, dist=d)
        args.update(kwargs)
        with pytest.raises(binding.IdkmError) as e:
            ctx.forward(W, C0, args["tau"], args["tol"], args["max_iter"], args["dist"])
        assert e.value.status == status
    with pytest.raises(binding.IdkmError) as e:  # empty input
        ctx.forward(torch.zeros((0, 1), dtype=torch.float32, device="cuda"), C0, 0.1, 1e-6, 5, d)
    assert e.value.status == 1
    with pytest.raises(binding.IdkmError) as e:  # k > m
        ctx.forward(dev(np.zeros((2, 1), dtype=np.float32)), dev(np.zeros((4, 1), dtype=np.float32)), 0.1, 1e-6, 5, d)
    assert e.value.status == 1
    with pytest.raises(binding.IdkmError) as e:  # d = 3 is not instantiated
        ctx.forward(dev(np.zeros((8, 3), dtype=np.float32)), dev(np.zeros((2, 3), dtype=np.float32)), 0.1, 1e-6, 5, d)
    assert e.value.status == 6
    # non-finite weights are reported, not propagated silently
    Wn = np.linspace(-1, 1, 64, dtype=np.float32).reshape(64, 1)
    Wn[5, 0] = np.nan
    with pytest.raises(binding.IdkmError) as e:
        ctx.forward(dev(Wn), dev(np.array([[-0.5], [0.5]], dtype=np.float32)), 0.1, 1e-6, 5, d)
    assert e.value.status == 4
    # alpha outside (0,1]
    ctx.forward(W + dev(np.arange(8, dtype=np.float32).reshape(8, 1)), dev(np.array([[1.0], [6.0]], dtype=np.float32)),
                1.0, 1e-6, 5, d)
    with pytest.raises(binding.IdkmError) as e:
        ctx.backward(W, binding.BWD_IMPLICIT, alpha=1.5)
    assert e.value.status == 1


# ---------------------------------------------------------------- minimal-residual (Krylov) backward

# (name, m, d, k, tau): k d <= 64 ends in one exact cycle; k d > 64 needs restarts.  The temperatures keep
# cond(I - dF/dC) below ~250 (float64 probe of these seeds), so that a float32 operator can reach the tolerance;
# in the last two cases the spectral radius of dF/dC exceeds 1 (the plain iteration diverges, the system is regular).
GMRES_CASES = [("k4d1", 70_001, 1, 4, 0.05), ("k16d1", 33_333, 1, 16, 0.005), ("k8d2", 20_011, 2, 8, 0.1),
               ("k3d1", 1_000, 1, 3, 0.1), ("k64d4", 4_003, 4, 64, 0.2), ("k100d2", 3_001, 2, 100, 0.01)]


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("name,m,d,k,tau", GMRES_CASES, ids=[c[0] for c in GMRES_CASES])
def test_krylov_backward_solves_the_linear_system_of_the_implicit_gradient(ctx, name, m, d, k, tau, dist):
    """g from IDKM_BWD_GMRES against the oracle's dense solve of (I - dF/dC*)^T g = v, the definition the
    averaged iteration converges to; dW against the oracle's backward with that g."""
    W, C0, G = _case(m, d, k, seed=300 + [c[0] for c in GMRES_CASES].index(name))
    Wd = dev(W)
    out = ctx.forward(Wd, dev(C0), tau, 1e-6, 60, dist, want_Wq=False)
    Cg = out["C"].cpu().numpy()
    Gd = dev(G)
    r = ctx.backward(Gd, binding.BWD_GMRES, tol=1e-6, max_iter=400)
    ref = orc.backward(W, Cg, tau, dist, G, "dense")
    assert r["info"].converged, r["info"]
    assert r["info"].residual <= 1e-6 * np.linalg.norm(ref["v"]) * 1.01
    assert rel(r["dW"].cpu().numpy(), ref["dW"]) < TOL_GRAD
    if k * d <= 64:
        assert r["info"].iters <= k * d + 1 + (k * d + 1)      # one exact cycle (+ at most one refinement cycle)
    # the solution itself, read back through one raw (dF/dC)^T pass at g_ref: J^T g_ref = g_ref - v
    u = ctx.step_JCT(dev(ref["g"].astype(np.float32))).cpu().numpy()
    assert rel(u, ref["g"] - ref["v"]) < TOL_GRAD
    # and the stream-path averaged iteration lands on the same dW wherever the oracle says it converges (spectral
    # radius of dF/dC* below one; two of the cases are chosen to have it above one)
    rho = float(np.abs(np.linalg.eigvals(orc.jacobian_C(Cg, W, tau, dist))).max())
    if rho < 0.97:
        ctx.set_path(binding.PATH_STREAM)
        try:
            it = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=1e-5, max_iter=3000, alpha=1.0)
        finally:
            ctx.set_path(binding.PATH_AUTO)
        assert it["info"].converged, (it["info"], rho)
        assert rel(r["dW"].cpu().numpy(), it["dW"].cpu().numpy()) < TOL_GRAD


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("cfg,m", [("C1", None), ("C3", 300_007), ("C2", 100_003), ("P16", 80_003), ("P16", 1_501)],
                         ids=["C1", "C3@300k", "C2@100k", "P16@80k", "P16@1.5k"])
def test_krylov_backward_inside_the_persistent_kernel(ctx, cfg, m, dist):
    """k d <= 64 with a team of one workgroup (C1, P16@1.5k) or a full-device team (two-level exchange): the whole
    minimal-residual solve runs in one launch.  Held to the oracle's dense solve and to the stream path's pass count."""
    p = wl.make_problem(cfg, dist, m=m)
    Wd, C0d = dev(p.W), dev(p.C0)
    out = ctx.forward(Wd, C0d, p.tau, p.tol, p.max_iter, dist)
    Cg = out["C"].cpu().numpy()
    G = p.G if p.G is not None else (2.0 * (orc.soft_quantize(p.W, Cg, p.tau, dist) - p.T)).astype(np.float32)
    Gd = dev(G)
    ref = orc.backward(p.W, Cg, p.tau, dist, G, "dense")
    res = {}
    for path in (binding.PATH_STREAM, binding.PATH_PERSISTENT):
        ctx.set_path(path)
        try:
            r = ctx.backward(Gd, binding.BWD_GMRES, tol=1e-5, max_iter=400)
        finally:
            ctx.set_path(binding.PATH_AUTO)
        assert r["info"].path == path
        res[path] = (r["info"], r["dW"].cpu().numpy(), ctx.get_cotangents(p.cfg.k, p.cfg.d)[1])
    (si, sdW, sg), (pi, pdW, pg) = res[binding.PATH_STREAM], res[binding.PATH_PERSISTENT]
    kd = p.cfg.k * p.cfg.d
    rho = float(np.abs(np.linalg.eigvals(orc.jacobian_C(Cg, p.W, p.tau, dist))).max())
    if rho < 0.97:
        # well conditioned: one exact cycle (+ the pass for the true residual) on either path
        assert pi.converged and si.converged and abs(pi.iters - si.iters) <= 2, (si, pi)
        assert pi.iters <= 2 * (kd + 1)
    # (otherwise -- C2 with the squared energy, condition number about 1e5 -- the float32 operator decides after how
    #  many restarts the true residual passes the test; both paths are held to the backward error below)
    # backward error of the returned g, evaluated by the oracle: || v + (dF/dC*)^T g - g || <= 1e-3 || v ||
    rr = ref["v"] + orc.vjp_F(Cg, p.W, p.tau, dist, pg)[0] - pg
    assert np.linalg.norm(rr) < TOL_GRAD * np.linalg.norm(ref["v"]), (np.linalg.norm(rr), np.linalg.norm(ref["v"]), pi)
    assert rel(pdW, sdW) < TOL_GRAD
    if rho < 0.97:  # well conditioned: the solution itself
        assert rel(pg, ref["g"]) < TOL_GRAD and rel(pdW, ref["dW"]) < TOL_GRAD
    ra = ctx.backward(Gd, binding.BWD_GMRES, tol=1e-5, max_iter=400)      # AUTO takes the persistent form here
    assert ra["info"].path == binding.PATH_PERSISTENT


def test_krylov_backward_on_the_persistent_path_is_refused(ctx):
    # (k = 3: the lane<->codeword family, whose persistent kernels do not hold the minimal-residual solve)
    W, C0, G = _case(5_000, 1, 3, seed=1)
    ctx.forward(dev(W), dev(C0), 0.05, 1e-6, 30, wl.DIST_SQL2)
    ctx.set_path(binding.PATH_PERSISTENT)
    with pytest.raises(binding.IdkmError) as e:
        ctx.backward(dev(G), binding.BWD_GMRES)
    ctx.set_path(binding.PATH_AUTO)
    assert e.value.status == 6
    r = ctx.backward(dev(G), binding.BWD_GMRES, tol=1e-6, max_iter=1)      # pass budget: ends unconverged or exact
    assert r["info"].iters <= 2


@pytest.mark.parametrize("dist", DISTS)
def test_krylov_backward_with_a_short_basis_restarts_and_still_converges(ctx, dist):
    name, m, d, k, tau = GMRES_CASES[2]      # k d = 16
    W, C0, G = _case(m, d, k, seed=302)
    out = ctx.forward(dev(W), dev(C0), tau, 1e-6, 60, dist, want_Wq=False)
    Cg = out["C"].cpu().numpy()
    ref = orc.backward(W, Cg, tau, dist, G, "dense")
    full = ctx.backward(dev(G), binding.BWD_GMRES, tol=1e-6, max_iter=400)
    ctx.set_gmres_basis(5)
    try:
        short = ctx.backward(dev(G), binding.BWD_GMRES, tol=1e-6, max_iter=400)
    finally:
        ctx.set_gmres_basis(64)
    assert short["info"].converged and full["info"].converged
    assert short["info"].iters > full["info"].iters            # several cycles of 5 + 1 passes
    assert rel(short["dW"].cpu().numpy(), ref["dW"]) < TOL_GRAD
    with pytest.raises(binding.IdkmError):
        ctx.set_gmres_basis(0)
    with pytest.raises(binding.IdkmError):
        ctx.set_gmres_basis(257)


@pytest.mark.parametrize("dist,tau", [(wl.DIST_L2, 1.0), (wl.DIST_SQL2, 8.0)])
def test_krylov_backward_at_the_largest_basis_vectors(ctx, dist, tau):
    """k d = 1024 (lane<->codeword family, the 1024-thread pass tail).  A dense oracle solve would need 1024 passes of
    the float64 oracle, so the reference is the oracle's own averaged iteration, run to 1e-9 where it converges fast
    (the temperatures are chosen for that)."""
    W, C0, G = wl.random_problem(3001, 4, 256, seed=333, std=0.5, spread=1.5)
    W, C0, G = W.astype(np.float32), C0.astype(np.float32), G.astype(np.float32)
    out = ctx.forward(dev(W), dev(C0), tau, 1e-6, 60, dist, want_Wq=False)
    Cg = out["C"].cpu().numpy()
    ref = orc.backward(W, Cg, tau, dist, G, "implicit", tol=1e-9, max_iter=300)
    assert ref["converged"]
    r = ctx.backward(dev(G), binding.BWD_GMRES, tol=1e-6, max_iter=300)
    assert r["info"].converged and r["info"].path == binding.PATH_STREAM
    assert r["info"].iters < ref["iters"] + 2
    assert rel(r["dW"].cpu().numpy(), ref["dW"]) < TOL_GRAD


def test_autograd_front_end_gives_the_oracle_gradient_of_a_loss(ctx):
    """L = sum((Wq - T)^2) through the autograd wrapper against the oracle's implicit gradient of the same loss."""
    from paper_2312_07759_amd.autograd import SoftKMeansQuantize
    W, C0, T = _case(20_011, 2, 8, seed=77)
    tau, dist = 0.1, wl.DIST_SQL2
    layer = SoftKMeansQuantize(tau, dist, tol=1e-7, max_iter=300, bwd_mode=binding.BWD_GMRES, bwd_tol=1e-7)
    Wt = dev(W).requires_grad_(True)
    Wq, Cstar = layer(Wt, dev(C0))
    loss = ((Wq - dev(T)) ** 2).sum()
    loss.backward()
    Cg = Cstar.cpu().numpy()
    G = (2.0 * (orc.soft_quantize(W, Cg, tau, dist) - T)).astype(np.float32)
    ref = orc.backward(W, Cg, tau, dist, G, "dense")
    assert layer.last_backward.converged
    assert rel(Wt.grad.cpu().numpy(), ref["dW"]) < TOL_GRAD
    assert not Cstar.requires_grad
    layer.close()


@pytest.mark.parametrize("path", ["stream", "persistent"])
@pytest.mark.parametrize("shape", [(30_011, 1, 4), (4_003, 4, 256)])
def test_results_do_not_change_when_the_sequence_numbers_wrap(path, shape):
    """The stamps of the exchanged words are 32-bit counters; just before they wrap the library clears its buffers and
    starts over.  The counters are advanced to that point and the same solve is repeated across it."""
    m, d, k = shape
    W, C0, G = _case(m, d, k, seed=4242)
    c = binding.Context(0)
    c.set_path(binding.PATH_STREAM if path == "stream" else binding.PATH_PERSISTENT)
    Wd, Cd, Gd = dev(W), dev(C0), dev(G)
    tau = 0.3 if d == 1 else 1.0

    def solve():
        f = c.forward(Wd, Cd, tau, 0.0, 20, wl.DIST_SQL2)
        b = c.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=15)
        return f["C"].clone(), f["Wq"].clone(), b["dW"].clone(), f["info"].iters, b["info"].iters

    first = solve()
    c.advance_sequence(0xFFFFFFFF)          # saturates a few hundred steps below the wrap
    for _ in range(40):                     # 40 x (21 + 17) exchanges or launches: well across it
        again = solve()
        assert again[3:] == first[3:]
        for x, y in zip(first[:3], again[:3]):
            assert torch.equal(x, y)
    c.close()


# More codewords than the data has clusters: in a soft solve the surplus codewords settle on (almost) the same points,
# so for many vectors the best and the second-best key differ by an ulp or not at all.  The integer result then hangs
# on the last bit of the key: it must be the documented expression -- every product and sum rounded on its own, in
# index order, lowest index on ties -- on every kernel family and path.
@pytest.mark.parametrize("m,d,k,clusters", [(300, 4, 256, 0), (500, 2, 100, 0), (20_000, 4, 16, 3), (20_000, 2, 8, 2),
                                            (5_000, 4, 200, 5), (3_000, 8, 32, 4)])
@pytest.mark.parametrize("path", [binding.PATH_STREAM, binding.PATH_PERSISTENT], ids=["stream", "persistent"])
def test_assignments_with_nearly_tied_keys(ctx, m, d, k, clusters, path):
    rng = np.random.default_rng(4242 + m + k)
    if clusters:
        centres = rng.standard_normal((clusters, d))
        W = centres[rng.integers(0, clusters, m)] + 0.05 * rng.standard_normal((m, d))
    else:
        W = 0.5 * rng.standard_normal((m, d))
    C0 = W[rng.choice(m, k, replace=False)] + 0.01 * rng.standard_normal((k, d))
    W, C0 = W.astype(np.float32), C0.astype(np.float32)
    ctx.set_path(path)
    try:
        for dist in DISTS:
            try:
                out = ctx.forward(dev(W), dev(C0), 0.3, 0.0, 25, dist, want_assign=True, want_Wq=False)
            except binding.IdkmError as e:
                assert path == binding.PATH_PERSISTENT and e.status == 6      # no persistent kernel for this shape
                continue
            Cg = out["C"].cpu().numpy()
            ref = orc.hard_assign_f32(W, Cg)
            got = out["assign"].cpu().numpy()
            np.testing.assert_array_equal(got, ref)
    finally:
        ctx.set_path(binding.PATH_AUTO)


def test_warm_start_and_temperature_schedule(ctx):
    # Alg. 2 solves the same layer again at every training step, and Sec. 6 suggests annealing the temperature: both
    # are sequences of ordinary calls in which C0 is the previous C* and tau changes.  Each stage is held to the oracle
    # from the same C0; the warm-started last stage must need fewer evaluations than a cold start at that temperature.
    cfg = wl.CONFIGS["C3"]
    p = wl.make_problem(cfg, wl.DIST_SQL2, m=100_003)
    W = p.W
    Wd = dev(W)
    C = p.C0.copy()
    rng = np.random.default_rng(11)
    stage_iters = []
    for stage, tau in enumerate([4 * p.tau, 2 * p.tau, p.tau, p.tau]):
        if stage == 3:
            # an SGD-like move of the weights (1 % of their spread) before the last solve
            W = (W + 1e-2 * W.std() * rng.standard_normal(W.shape)).astype(np.float32)
            Wd = dev(W)
        out = ctx.forward(Wd, dev(C), tau, p.tol, p.max_iter, wl.DIST_SQL2, want_Wq=False)
        ref = orc.soft_kmeans(W, C, tau, p.tol, p.max_iter, wl.DIST_SQL2)
        Cg = out["C"].cpu().numpy()
        assert out["info"].converged and ref["converged"]
        assert abs(out["info"].iters - ref["iters"]) <= 1
        assert rel(Cg, ref["C"]) < TOL_VAL
        stage_iters.append(out["info"].iters)
        C = Cg
    cold = ctx.forward(Wd, dev(p.C0), p.tau, p.tol, p.max_iter, wl.DIST_SQL2, want_Wq=False)
    assert stage_iters[-1] < cold["info"].iters


# The widest shapes of the lane<->vector family (k d >= 32, d >= 2) take h_j . (w - F*_j) apart into h_j . (w - mu)
# and a per-codeword constant in their (dF/dC)^T and last passes.  With a layer a hundred spreads away from the origin
# the two parts would be large and nearly equal if mu were not the centre of the codebook.  The scalar shapes work in
# scaled coordinates (w - c_0) s - (c_j - c_0) s in their backward passes, for the same reason relative to a codeword.
@pytest.mark.parametrize("path", [binding.PATH_STREAM, binding.PATH_PERSISTENT], ids=["stream", "persistent"])
@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("k,d", [(16, 4), (8, 4), (16, 2), (4, 2), (2, 2), (4, 4), (4, 1), (16, 1)])
def test_backward_of_a_layer_far_from_the_origin(ctx, k, d, dist, path):
    rng = np.random.default_rng(770 + 16 * k + d)
    m = 20_011
    W = (5.0 + 0.05 * rng.standard_normal((m, d))).astype(np.float32)
    C0 = (W[rng.choice(m, k, replace=False)] + 0.002 * rng.standard_normal((k, d))).astype(np.float32)
    G = rng.standard_normal((m, d)).astype(np.float32)
    tau = 1e-3 if dist == wl.DIST_SQL2 else 1e-2
    ctx.set_path(path)
    try:
        out = ctx.forward(dev(W), dev(C0), tau, 0.0, 25, dist)
        assert out["info"].path == path
        Cg = out["C"].cpu().numpy()
        assert rel(Cg, orc.soft_kmeans(W, C0, tau, 0.0, 25, dist)["C"]) < TOL_VAL
        Gd = dev(G)
        bj = ctx.backward(Gd, binding.BWD_JFB)
        assert rel(bj["dW"].cpu().numpy(), orc.backward(W, Cg, tau, dist, G, "jfb")["dW"]) < TOL_GRAD
        bi = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=12, alpha=1.0)
        ri = orc.backward(W, Cg, tau, dist, G, "implicit", tol=0.0, max_iter=12, alpha=1.0)
        assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD
    finally:
        ctx.set_path(binding.PATH_AUTO)


# Squared energy, d >= 2: the forward loop and the (dF/dC)^T pass take the exponents of the row softmax as products about
# the mean codeword; their rounding error is a few float32 ulps of s^2 |c - mu| |w - mu|, s^2 = log2(e)/tau.  The lower
# the temperature against the spread of the codebook, the larger that is: here s^2 |c - mu|^2 runs from about 250 to
# 6000 (rows from soft to nearly hard).
@pytest.mark.parametrize("path", [binding.PATH_STREAM, binding.PATH_PERSISTENT], ids=["stream", "persistent"])
@pytest.mark.parametrize("tau", [0.05, 0.01, 0.002])
@pytest.mark.parametrize("k,d", [(16, 4), (4, 2), (8, 2)])
def test_product_form_of_the_exponents_from_soft_to_nearly_hard_rows(ctx, k, d, tau, path):
    W, C0, G = wl.random_problem(30_011, d, k, seed=900 + k + d, std=0.5, spread=1.5)
    W, G = W.astype(np.float32), G.astype(np.float32)
    C0 = (C0 + 0.05 * np.random.default_rng(5).standard_normal(C0.shape)).astype(np.float32)
    dist = wl.DIST_SQL2
    ctx.set_path(path)
    try:
        out = ctx.forward(dev(W), dev(C0), tau, 0.0, 6, dist)
        Cg = out["C"].cpu().numpy()
        ref = orc.soft_kmeans(W, C0, tau, 0.0, 6, dist)
        assert rel(Cg, ref["C"]) < TOL_VAL, rel(Cg, ref["C"])
        assert np.abs(Cg - ref["C"]).max() < TOL_VAL * np.abs(ref["C"]).max()
        bi = ctx.backward(dev(G), binding.BWD_IMPLICIT, tol=0.0, max_iter=8, alpha=1.0)
        ri = orc.backward(W, Cg, tau, dist, G, "implicit", tol=0.0, max_iter=8, alpha=1.0)
        if not (bi["info"].converged or ri["converged"]):
            assert bi["info"].iters == ri["iters"] and bi["info"].alpha == ri["alpha"]
        assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD, rel(bi["dW"].cpu().numpy(), ri["dW"])
        v, g = ctx.get_cotangents(k, d)
        assert rel(g, ri["g"]) < TOL_GRAD, rel(g, ri["g"])
    finally:
        ctx.set_path(binding.PATH_AUTO)


# Plain norm, scalar weights: d e / d w is the sign of w - c, and zero where the two coincide exactly.  The backward
# passes work in scaled coordinates (w - c_0) s - (c_j - c_0) s; the two products have to be rounded on their own, or a
# weight that equals a codeword would come out with the sign of a rounding residual.  Here a tenth (k = 4) to two
# fifths (k = 16) of the weights sit exactly on codewords: a sign in place of the zero would move the result by 7-12 %.
@pytest.mark.parametrize("k", [4, 16])
def test_scalar_weights_that_coincide_with_codewords_plain_norm(ctx, k):
    rng = np.random.default_rng(31)
    m = 50_000
    grid = np.linspace(-1, 1, 41).astype(np.float32)
    W = rng.choice(grid, m).astype(np.float32).reshape(m, 1)
    C = np.sort(rng.choice(grid, k, replace=False)).astype(np.float32).reshape(k, 1)
    g = rng.standard_normal((k, 1)).astype(np.float32)
    assert np.isin(W, C).mean() > 0.05
    ctx.step_F(dev(W), dev(C), 0.2, wl.DIST_L2)
    u = ctx.step_JCT(dev(g)).cpu().numpy()
    assert rel(u, orc.vjp_F(C, W, 0.2, wl.DIST_L2, g)[0]) < TOL_GRAD
    # the whole backward from this codebook (one evaluation of F moves it off the grid; the first pass, for v, and
    # the last, for dW, still see it where the forward left it only through F*: compare at the GPU's own C*)
    for path in (binding.PATH_STREAM, binding.PATH_PERSISTENT):
        ctx.set_path(path)
        try:
            out = ctx.forward(dev(W), dev(C), 0.2, 0.0, 1, wl.DIST_L2)
            Cg = out["C"].cpu().numpy()
            G = rng.standard_normal((m, 1)).astype(np.float32)
            bi = ctx.backward(dev(G), binding.BWD_IMPLICIT, tol=0.0, max_iter=6, alpha=1.0)
            ri = orc.backward(W, Cg, 0.2, wl.DIST_L2, G, "implicit", tol=0.0, max_iter=6, alpha=1.0)
            assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD
        finally:
            ctx.set_path(binding.PATH_AUTO)
