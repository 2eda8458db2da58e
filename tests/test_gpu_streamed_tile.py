"""Persistent solves whose share of W does not stay in LDS (lane<->vector family): every pass reads it from memory with
16-byte loads.  The form is forced on small layers through idkm_set_tile_limit(0), so that ragged ends (sizes that
are no multiple of the vectors per load, workgroups with fewer vectors than threads), every (k, d) and all backward
modes are compared with the oracle at sizes it finishes quickly; one case is large enough to take the form by itself.  (Under IDKM_PATH_AUTO such layers go to the stream path,
which is as fast; the persistent form is for callers that want one launch per solve.)
Bars as everywhere: C*, Wq 1e-4; gradients 1e-3; hard assignments bit-exact on the kernel's own C*."""
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


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    c.set_path(binding.PATH_PERSISTENT)
    c.set_tile_limit(0)
    yield c
    c.close()


SHAPES = [(k, d) for k in (2, 4, 8, 16) for d in (1, 2, 4)]


@pytest.mark.parametrize("dist", [wl.DIST_SQL2, wl.DIST_L2], ids=["sql2", "l2"])
@pytest.mark.parametrize("k,d", SHAPES, ids=[f"k{k}d{d}" for k, d in SHAPES])
def test_forward_and_backward(ctx, k, d, dist):
    m = 40_000 + 37 * k + d          # not a multiple of 4: the last workgroup ends inside a 16-byte group
    W, C0, G = wl.random_problem(m, d, k, seed=5000 + 16 * k + d, std=0.5, spread=1.5)
    W, G = W.astype(np.float32), G.astype(np.float32)
    C0 = (C0 + 0.01 * np.random.default_rng(k).standard_normal(C0.shape)).astype(np.float32)
    tau, iters = 0.15, 20
    out = ctx.forward(dev(W), dev(C0), tau, 0.0, iters, dist, want_assign=True)
    assert out["info"].path == binding.PATH_PERSISTENT and out["info"].iters == iters
    ref = orc.soft_kmeans(W, C0, tau, 0.0, iters, dist)
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, ref["C"]) < TOL_VAL
    assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(W, Cg, tau, dist)) < TOL_VAL
    assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(W, Cg))
    Gd = dev(G)
    bj = ctx.backward(Gd, binding.BWD_JFB)
    assert rel(bj["dW"].cpu().numpy(), orc.backward(W, Cg, tau, dist, G, "jfb")["dW"]) < TOL_GRAD
    bi = ctx.backward(Gd, binding.BWD_IMPLICIT, tol=0.0, max_iter=12, alpha=1.0)
    ri = orc.backward(W, Cg, tau, dist, G, "implicit", tol=0.0, max_iter=12, alpha=1.0)
    assert bi["info"].path == binding.PATH_PERSISTENT
    assert rel(bi["dW"].cpu().numpy(), ri["dW"]) < TOL_GRAD
    if k * d * (k * d + d + 1) <= 32:
        bd = ctx.backward(Gd, binding.BWD_DENSE)
        assert bd["info"].path == binding.PATH_PERSISTENT
        assert rel(bd["dW"].cpu().numpy(), orc.backward(W, Cg, tau, dist, G, "dense")["dW"]) < TOL_GRAD


@pytest.mark.parametrize("m", [2, 5, 255, 257, 1027, 70_001])
def test_small_and_ragged_sizes(ctx, m):
    k, d = (4, 1) if m >= 4 else (2, 1)
    W, C0, _ = wl.random_problem(m, d, k, seed=6000 + m, std=0.5, spread=1.5)
    W, C0 = W.astype(np.float32), C0.astype(np.float32)
    out = ctx.forward(dev(W), dev(C0), 0.2, 0.0, 10, wl.DIST_SQL2, want_assign=True)
    ref = orc.soft_kmeans(W, C0, 0.2, 0.0, 10, wl.DIST_SQL2)
    Cg = out["C"].cpu().numpy()
    assert rel(Cg, ref["C"]) < TOL_VAL
    assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(W, Cg, 0.2, wl.DIST_SQL2)) < TOL_VAL
    assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(W, Cg))


def test_unaligned_tensors_take_the_stream_path():
    c = binding.Context(0)
    try:
        c.set_tile_limit(0)
        c.set_path(binding.PATH_PERSISTENT)
        W, C0, _ = wl.random_problem(30_001, 1, 4, seed=61, std=0.5, spread=1.5)
        buf = torch.zeros(30_002, 1, dtype=torch.float32, device="cuda")
        Wd = buf[1:]                                         # 4 bytes past a 16-byte boundary
        Wd.copy_(dev(W))
        with pytest.raises(binding.IdkmError):               # the persistent path cannot serve it ...
            c.forward(Wd, dev(C0), 0.2, 0.0, 10, wl.DIST_SQL2)
        c.set_path(binding.PATH_AUTO)                        # ... the default falls back to the stream path
        out = c.forward(Wd, dev(C0), 0.2, 0.0, 10, wl.DIST_SQL2)
        assert out["info"].path == binding.PATH_STREAM
        ref = orc.soft_kmeans(W.astype(np.float32), C0.astype(np.float32), 0.2, 0.0, 10, wl.DIST_SQL2)
        assert rel(out["C"].cpu().numpy(), ref["C"]) < TOL_VAL
    finally:
        c.close()


def test_layer_larger_than_the_chip():
    # 10.5 M scalars: more than the 256 workgroups can hold in LDS (about 9.4 M), default tile limit
    c = binding.Context(0)
    try:
        c.set_path(binding.PATH_PERSISTENT)
        cfg = wl.CONFIGS["C3"]
        p = wl.make_problem(cfg, wl.DIST_SQL2, m=10_500_003)
        Wd, Cd = dev(p.W), dev(p.C0)
        out = c.forward(Wd, Cd, p.tau, p.tol, 12, wl.DIST_SQL2, want_assign=True)
        assert out["info"].path == binding.PATH_PERSISTENT
        ref = orc.soft_kmeans(p.W, p.C0, p.tau, p.tol, 12, wl.DIST_SQL2)
        Cg = out["C"].cpu().numpy()
        assert rel(Cg, ref["C"]) < TOL_VAL and out["info"].iters == ref["iters"]
        assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(p.W, Cg))
        G = np.random.default_rng(3).standard_normal(p.W.shape).astype(np.float32) * 1e-4
        bj = c.backward(dev(G), binding.BWD_JFB)
        assert bj["info"].path == binding.PATH_PERSISTENT
        assert rel(bj["dW"].cpu().numpy(), orc.backward(p.W, Cg, p.tau, wl.DIST_SQL2, G, "jfb")["dW"]) < TOL_GRAD
        # translation identity of the implicit gradient (holds at any size): sum_i dL/dW_i = sum_i G_i
        bd = c.backward(dev(G), binding.BWD_DENSE)
        assert bd["info"].path == binding.PATH_PERSISTENT
        s_dw = bd["dW"].double().sum().item()
        assert abs(s_dw - float(G.astype(np.float64).sum())) < 1e-3 * float(np.abs(G).astype(np.float64).sum())
    finally:
        c.close()
