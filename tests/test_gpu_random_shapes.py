"""Seeded sweep over shapes the named parity cases do not list: every (k, d) the lane<->vector family instantiates,
odd k and ragged m for the lane<->codeword family, both energies, both scheduling paths where offered.  Same bars as
the named cases: C*, Wq 1e-4; gradients 1e-3 (norm-wise, against the float64 oracle at the kernel's own C*)."""
import numpy as np
import pytest
import torch

from oracle import idkm_oracle as orc
from paper_2312_07759_amd import binding
from paper_2312_07759_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL_VAL, TOL_GRAD = 1e-4, 1e-3


def rel(x, ref):
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / (den if den > 0 else 1.0))


def dev(x):
    return torch.as_tensor(np.ascontiguousarray(x), dtype=torch.float32).cuda()


def _cases():
    rng = np.random.default_rng(20231207)
    out = []
    small = [(k, d) for k in (2, 4, 8, 16) for d in (1, 2, 4)]
    lane = [(3, 1), (5, 2), (24, 4), (64, 2), (65, 1), (96, 4), (130, 2), (200, 1), (17, 8), (40, 8)]
    for k, d in small + lane:
        m = int(rng.integers(max(2 * k, 300), 9000))
        tau = float(rng.choice([0.05, 0.15, 0.5]))
        out.append((k, d, m, tau, int(rng.integers(0, 1 << 30))))
    return out


CASES = _cases()


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("dist", [wl.DIST_L2, wl.DIST_SQL2])
@pytest.mark.parametrize("k,d,m,tau,seed", CASES, ids=[f"k{c[0]}d{c[1]}m{c[2]}" for c in CASES])
def test_forward_and_backward_on_both_paths(ctx, k, d, m, tau, seed, dist):
    W, C0, G = wl.random_problem(m, d, k, seed=seed, std=0.5, spread=1.5)
    W, G = W.astype(np.float32), G.astype(np.float32)
    C0 = (C0 + 0.01 * np.random.default_rng(seed + 1).standard_normal(C0.shape)).astype(np.float32)
    Wd, Cd, Gd = dev(W), dev(C0), dev(G)
    iters = 25
    ref = orc.soft_kmeans(W, C0, tau, 0.0, iters, dist)
    tried = 0
    for path in (binding.PATH_STREAM, binding.PATH_PERSISTENT):
        ctx.set_path(path)
        try:
            try:
                out = ctx.forward(Wd, Cd, tau, 0.0, iters, dist, want_assign=True)
            except binding.IdkmError as e:
                assert path == binding.PATH_PERSISTENT and e.status == 6      # no persistent kernel for this shape
                continue
            tried += 1
            Cg = out["C"].cpu().numpy()
            assert out["info"].iters == iters and out["info"].path == path
            assert rel(Cg, ref["C"]) < TOL_VAL, (path, rel(Cg, ref["C"]))
            assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(W, Cg, tau, dist)) < TOL_VAL
            assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(W, Cg))
            bj = ctx.backward(Gd, binding.BWD_JFB)
            assert rel(bj["dW"].cpu().numpy(), orc.backward(W, Cg, tau, dist, G, "jfb")["dW"]) < TOL_GRAD
            bi = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=12, alpha=1.0)
            ri = orc.backward(W, Cg, tau, dist, G, "implicit", tol=0.0, max_iter=12, alpha=1.0)
            if not (bi["info"].converged or ri["converged"]):      # an exactly zero step ends either side early
                assert bi["info"].iters == ri["iters"] and bi["info"].alpha == ri["alpha"]
            assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD, (path, rel(bi["dW"].cpu().numpy(), ri["dW"]))
        finally:
            ctx.set_path(binding.PATH_AUTO)
    assert tried >= 1


def _team_cases():
    """Layers large enough for teams of 8 to 256 workgroups (the two-level grid exchange), ragged sizes."""
    rng = np.random.default_rng(20231208)
    out = []
    for k in (2, 4, 8, 16):
        for d in (1, 2, 4):
            m = int(rng.integers(64 * 1024 + 1, 300_000))
            out.append((k, d, m, float(rng.choice([0.05, 0.15, 0.5])), int(rng.integers(0, 1 << 30))))
    out.append((4, 1, 64 * 1024 - 1023, 0.1, 7))   # exactly 64 workgroups
    out.append((4, 1, 65 * 1024 + 5, 0.1, 8))      # 66 workgroups: dies with 9 and with 8 members
    out.append((2, 2, 255 * 1024 + 3, 0.1, 9))     # 256 workgroups, the last one nearly empty
    out.append((4, 1, 7 * 1024 + 1, 0.1, 10))      # 8 workgroups: the smallest team of the two-level exchange, one per die
    out.append((8, 2, 4_099, 0.1, 14))             # just above one workgroup's share: 8 workgroups of 513 vectors
    out.append((4, 1, 9 * 1024 + 5, 0.1, 11))      # 10 workgroups: dies with two members and with one
    out.append((16, 4, 20 * 1024 + 3, 0.15, 12))   # 21 workgroups, 80 sums per workgroup
    out.append((2, 2, 36 * 1024 + 7, 0.1, 13))     # 37 workgroups
    return out


TEAM_CASES = _team_cases()


@pytest.mark.parametrize("dist", [wl.DIST_L2, wl.DIST_SQL2])
@pytest.mark.parametrize("k,d,m,tau,seed", TEAM_CASES, ids=[f"k{c[0]}d{c[1]}m{c[2]}" for c in TEAM_CASES])
def test_full_device_teams_on_the_persistent_path(ctx, k, d, m, tau, seed, dist):
    W, C0, G = wl.random_problem(m, d, k, seed=seed, std=0.5, spread=1.5)
    W, G = W.astype(np.float32), G.astype(np.float32)
    C0 = (C0 + 0.01 * np.random.default_rng(seed + 1).standard_normal(C0.shape)).astype(np.float32)
    Wd, Cd, Gd = dev(W), dev(C0), dev(G)
    iters = 8
    ref = orc.soft_kmeans(W, C0, tau, 0.0, iters, dist)
    out = ctx.forward(Wd, Cd, tau, 0.0, iters, dist, want_assign=True)
    assert out["info"].iters == iters and out["info"].path == binding.PATH_PERSISTENT
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, ref["C"]) < TOL_VAL, rel(Cg, ref["C"])
    assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(W, Cg, tau, dist)) < TOL_VAL
    assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(W, Cg))
    bj = ctx.backward(Gd, binding.BWD_JFB)
    rj = orc.backward(W, Cg, tau, dist, G, "jfb")
    assert rel(bj["dW"].cpu().numpy(), rj["dW"]) < TOL_GRAD
    v, g = ctx.get_cotangents(k, d)
    assert rel(v, rj["v"]) < TOL_GRAD
    bi = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=6, alpha=1.0)
    ri = orc.backward(W, Cg, tau, dist, G, "implicit", tol=0.0, max_iter=6, alpha=1.0)
    if not (bi["info"].converged or ri["converged"]):
        assert bi["info"].iters == ri["iters"] and bi["info"].alpha == ri["alpha"]
    assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD, rel(bi["dW"].cpu().numpy(), ri["dW"])
    if k * d <= 64:      # (every case: the minimal-residual solve inside the persistent kernel, basis of up to k d vectors)
        bg = ctx.backward(Gd, binding.BWD_GMRES, tol=1e-5, max_iter=200)
        assert bg["info"].path == binding.PATH_PERSISTENT
        gg = ctx.get_cotangents(k, d)[1]
        res = rj["v"] + orc.vjp_F(Cg, W, tau, dist, gg)[0] - gg
        assert np.linalg.norm(res) < TOL_GRAD * np.linalg.norm(rj["v"]), (bg["info"], np.linalg.norm(res), np.linalg.norm(rj["v"]))
