"""Pins for the derivative half of the CPU oracle (Sec. 4.2 implicit gradient, Sec. 4.3 JFB).

Independent checks only: central finite differences of the oracle's own forward
map, an autodiff (PyTorch CPU, float64) of the *matrix form* of F written with
library softmax/cdist, the dense linear solve, structural identities.
"""
import numpy as np
import pytest
import torch

from oracle import idkm_oracle as orc
from paper_2312_07759_amd import workloads as wl

DISTS = [orc.DIST_L2, orc.DIST_SQL2]
CASES = [(40, 1, 3), (36, 2, 4), (30, 4, 5)]


def _problem(m, d, k, seed):
    W, C0, G = wl.random_problem(m, d, k, seed=seed, std=0.45, spread=1.6)
    # C0 is drawn from the rows of W; move it off them, the plain norm is not differentiable at w == c
    C0 = C0 + 0.05 * np.random.default_rng(seed + 1).standard_normal(C0.shape)
    return W, C0, G


def _F_torch(C, W, tau, dist):
    """Matrix form of Eq. "deepeqc" with library routines: diag(A^T 1)^-1 A^T W, A = rowsoftmax(-D/tau)."""
    if dist == orc.DIST_L2:
        D = torch.cdist(W, C)
    else:
        D = (W[:, None, :] - C[None, :, :]).pow(2).sum(-1)
    A = torch.softmax(-D / tau, dim=1)
    return (A.T @ W) / A.sum(0)[:, None], A


def _loss_torch(W, C, tau, dist, T):
    _, A = _F_torch(C, W, tau, dist)
    return ((A @ C - T) ** 2).sum()


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("m,d,k", CASES)
def test_vjp_F_matches_central_differences_of_F(dist, m, d, k):
    W, C0, _ = _problem(m, d, k, 100 + d)
    tau = 0.35
    g = np.random.default_rng(7).standard_normal((k, d))
    JCg, JWg = orc.vjp_F(C0, W, tau, dist, g)
    eps = 1e-6
    fd_C = np.zeros_like(C0)
    for j in range(k):
        for r in range(d):
            Cp, Cm = C0.copy(), C0.copy()
            Cp[j, r] += eps
            Cm[j, r] -= eps
            fd_C[j, r] = ((orc.F(Cp, W, tau, dist) - orc.F(Cm, W, tau, dist)) * g).sum() / (2 * eps)
    fd_W = np.zeros_like(W)
    for i in range(m):
        for r in range(d):
            Wp, Wm = W.copy(), W.copy()
            Wp[i, r] += eps
            Wm[i, r] -= eps
            fd_W[i, r] = ((orc.F(C0, Wp, tau, dist) - orc.F(C0, Wm, tau, dist)) * g).sum() / (2 * eps)
    np.testing.assert_allclose(JCg, fd_C, rtol=2e-7, atol=2e-8)
    np.testing.assert_allclose(JWg, fd_W, rtol=2e-7, atol=2e-8)


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("m,d,k", CASES)
def test_vjp_F_and_loss_cotangents_match_autodiff_of_the_matrix_form(dist, m, d, k):
    W, C0, G = _problem(m, d, k, 200 + d)
    tau = 0.3
    g = np.random.default_rng(8).standard_normal((k, d))
    Wt = torch.tensor(W, requires_grad=True)
    Ct = torch.tensor(C0, requires_grad=True)
    Fv, A = _F_torch(Ct, Wt, tau, dist)
    gC, gW = torch.autograd.grad((Fv * torch.tensor(g)).sum(), [Ct, Wt])
    JCg, JWg = orc.vjp_F(C0, W, tau, dist, g)
    np.testing.assert_allclose(JCg, gC.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(JWg, gW.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(orc.attention(W, C0, tau, dist), A.detach().numpy(), rtol=1e-12, atol=1e-15)
    # loss cotangents at fixed upstream G
    Fv, A = _F_torch(Ct, Wt, tau, dist)
    vC, vW = torch.autograd.grad(((A @ Ct) * torch.tensor(G)).sum(), [Ct, Wt])
    v, direct = orc.loss_cotangents(W, C0, tau, dist, G)
    np.testing.assert_allclose(v, vC.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(direct, vW.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("dist", DISTS)
def test_translation_identity_of_the_jacobians(dist):
    # F(C+t, W+t) = F(C, W)+t  =>  summing a VJP over all rows of C and W returns the summed cotangent
    W, C0, _ = _problem(50, 3, 4, 300)
    g = np.random.default_rng(9).standard_normal((4, 3))
    JCg, JWg = orc.vjp_F(C0, W, 0.4, dist, g)
    np.testing.assert_allclose(JCg.sum(0) + JWg.sum(0), g.sum(0), rtol=1e-11, atol=1e-12)


def test_squared_energy_jacobian_is_symmetrisable_with_spectrum_in_0_1():
    W, C0, _ = _problem(300, 2, 4, 310)
    tau = 0.5
    out = orc.soft_kmeans(W, C0, tau, 1e-13, 20000, orc.DIST_SQL2)
    assert out["converged"]
    C = out["C"]
    J = orc.jacobian_C(C, W, tau, orc.DIST_SQL2)
    n = orc.mstep(orc.attention(W, C, tau, orc.DIST_SQL2), W, C)[1]
    N = np.kron(np.diag(n), np.eye(2))
    S = N @ (np.eye(8) - J)
    np.testing.assert_allclose(S, S.T, rtol=0, atol=1e-9 * np.abs(S).max())
    ev = np.linalg.eigvals(J)
    assert np.abs(ev.imag).max() < 1e-9 and ev.real.min() > -1e-9 and ev.real.max() < 1.0


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("m,d,k", [(40, 1, 3), (36, 2, 3)])
def test_implicit_gradient_matches_finite_differences_of_the_solved_layer(dist, m, d, k):
    W, C0, _ = _problem(m, d, k, 400 + d)
    T = np.random.default_rng(10).standard_normal((m, d)) * 0.5
    tau = 0.3

    def layer_loss(Wx):
        out = orc.soft_kmeans(Wx, C0, tau, 1e-14, 50000, dist)
        assert out["converged"]
        return float(((orc.soft_quantize(Wx, out["C"], tau, dist) - T) ** 2).sum()), out["C"]

    L0, Cs = layer_loss(W)
    G = 2.0 * (orc.soft_quantize(W, Cs, tau, dist) - T)
    dense = orc.backward(W, Cs, tau, dist, G, "dense")
    it = orc.backward(W, Cs, tau, dist, G, "implicit", tol=1e-13, max_iter=20000, alpha=1.0)
    assert it["converged"]
    np.testing.assert_allclose(it["dW"], dense["dW"], rtol=1e-9, atol=1e-10)
    eps = 1e-5
    rng = np.random.default_rng(12)
    coords = [(int(rng.integers(m)), int(rng.integers(d))) for _ in range(12)]
    for (i, r) in coords:
        Wp, Wm = W.copy(), W.copy()
        Wp[i, r] += eps
        Wm[i, r] -= eps
        fd = (layer_loss(Wp)[0] - layer_loss(Wm)[0]) / (2 * eps)
        assert abs(fd - dense["dW"][i, r]) <= 2e-6 * max(1.0, abs(fd)), (i, r, fd, dense["dW"][i, r])
    # translation invariance of the whole layer: the implicit gradient sums to the upstream sum ...
    np.testing.assert_allclose(dense["dW"].sum(0), G.sum(0), rtol=1e-9, atol=1e-9)
    # ... and the one-step approximation does not
    jfb = orc.backward(W, Cs, tau, dist, G, "jfb")
    assert np.abs(jfb["dW"].sum(0) - G.sum(0)).max() > 1e-3


@pytest.mark.parametrize("dist", DISTS)
def test_unrolled_autodiff_converges_to_the_implicit_gradient(dist):
    # The DKM computation: reverse mode through T stored iterations (Sec. 3.3).  As T grows it tends
    # to the implicit gradient, which needs none of them.
    W, C0, _ = _problem(60, 2, 3, 500)
    T = np.random.default_rng(13).standard_normal((60, 2)) * 0.5
    tau = 0.3
    out = orc.soft_kmeans(W, C0, tau, 1e-14, 50000, dist)
    Cs = out["C"]
    G = 2.0 * (orc.soft_quantize(W, Cs, tau, dist) - T)
    ref = orc.backward(W, Cs, tau, dist, G, "dense")["dW"]
    errs = []
    for steps in (5, 40, 400):
        Wt = torch.tensor(W, requires_grad=True)
        C = torch.tensor(C0)
        for _ in range(steps):
            C = _F_torch(C, Wt, tau, dist)[0]
        (gW,) = torch.autograd.grad(_loss_torch(Wt, C, tau, dist, torch.tensor(T)), [Wt])
        errs.append(np.linalg.norm(gW.numpy() - ref) / np.linalg.norm(ref))
    assert errs[0] > errs[1] > errs[2] or errs[1] < 1e-9
    assert errs[2] < 1e-8


@pytest.mark.parametrize("dist", DISTS)
def test_jfb_and_neumann_truncations_equal_unrolling_from_the_detached_solution(dist):
    # Sec. 4.3: starting Alg. 1 at C* and differentiating T steps gives the T-term Neumann truncation;
    # T = 1 is JFB.
    W, C0, _ = _problem(60, 2, 3, 600)
    T = np.random.default_rng(14).standard_normal((60, 2)) * 0.5
    tau = 0.3
    Cs = orc.soft_kmeans(W, C0, tau, 1e-14, 50000, dist)["C"]
    G = 2.0 * (orc.soft_quantize(W, Cs, tau, dist) - T)
    for steps in (1, 2, 5):
        Wt = torch.tensor(W, requires_grad=True)
        C = torch.tensor(Cs)
        for _ in range(steps):
            C = _F_torch(C, Wt, tau, dist)[0]
        (gW,) = torch.autograd.grad(_loss_torch(Wt, C, tau, dist, torch.tensor(T)), [Wt])
        if steps == 1:
            mine = orc.backward(W, Cs, tau, dist, G, "jfb")["dW"]
        else:
            mine = orc.backward(W, Cs, tau, dist, G, "implicit", tol=0.0, max_iter=steps - 1, alpha=1.0)["dW"]
        np.testing.assert_allclose(mine, gW.numpy(), rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("dist", DISTS)
def test_damping_does_not_change_the_solution_and_matrix_iteration_agrees(dist):
    W, C0, G = _problem(80, 1, 4, 700)
    tau = 0.25
    Cs = orc.soft_kmeans(W, C0, tau, 1e-14, 50000, dist)["C"]
    v, _ = orc.loss_cotangents(W, Cs, tau, dist, G)
    dense = orc.solve_dense(Cs, W, tau, dist, v)
    for alpha in (1.0, 0.5, 0.25):
        s = orc.solve_iterative(Cs, W, tau, dist, v, 1e-13, 100000, alpha)
        assert s["converged"] and s["alpha"] == alpha
        np.testing.assert_allclose(s["g"], dense, rtol=1e-9, atol=1e-10)
    # the paper's matrix iteration for M* = (I - dF/dC)^-1 with alpha = .25 solves the same system
    J = orc.jacobian_C(Cs, W, tau, dist)
    M, _ = orc.inverse_matrix_iteration(J, alpha=0.25)
    np.testing.assert_allclose(M, np.linalg.inv(np.eye(4) - J), rtol=1e-8, atol=1e-9)
    np.testing.assert_allclose(M.T @ v.reshape(-1), dense.reshape(-1), rtol=1e-8, atol=1e-9)


def test_divergent_iteration_restarts_with_halved_alpha():
    # A linear system whose Jacobian has an eigenvalue below -1: plain iteration diverges, damping converges.
    # Driven through the same routine by substituting a linear map for vjp_F.
    J = np.array([[-1.6, 0.0], [0.0, 0.3]])
    v = np.array([[1.0], [1.0]])
    saved = orc.vjp_F
    try:
        orc.vjp_F = lambda C, W, tau, dist, g: ((J.T @ g.reshape(-1)).reshape(g.shape), None)
        s = orc.solve_iterative(None, None, 1.0, 0, v, 1e-12, 10000, alpha=1.0)
    finally:
        orc.vjp_F = saved
    assert s["converged"] and s["alpha"] == 0.5
    np.testing.assert_allclose(s["g"].reshape(-1), np.linalg.solve(np.eye(2) - J.T, v.reshape(-1)), rtol=1e-10)


@pytest.mark.parametrize("dist", DISTS)
def test_jfb_tends_to_implicit_for_well_separated_clusters(dist):
    W, C0, G = wl.random_problem(90, 2, 3, seed=800, std=0.05, spread=3.0)
    # start from one point of each blob so no cluster is shared
    tau = 0.02
    Cs = orc.soft_kmeans(W, C0, tau, 1e-14, 5000, dist)["C"]
    a = orc.backward(W, Cs, tau, dist, G, "dense")["dW"]
    b = orc.backward(W, Cs, tau, dist, G, "jfb")["dW"]
    J = orc.jacobian_C(Cs, W, tau, dist)
    if np.abs(np.linalg.eigvals(J)).max() < 1e-6:
        np.testing.assert_allclose(a, b, rtol=1e-4, atol=1e-8)
    else:  # blobs merged for this seed: JFB is only an approximation then
        assert np.linalg.norm(a - b) / np.linalg.norm(a) < 1.0
