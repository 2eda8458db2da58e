"""Batched per-layer calls (the layer loops of Alg. 2) against the oracle and against the per-layer entry points.

Every layer of a batch is an independent problem, so each result is held to the same bar as a single call:
C*, Wq within 1e-4, gradients within 1e-3 of the float64 oracle (norm-wise relative), hard assignments bit-exact
against the float32 key evaluated on the kernel's own C*.  Between the batched and the per-layer launch forms the
arithmetic is the same source with the same team sizes and summation orders; the two kernels are scheduled
differently (a batched workgroup shares its SIMDs, so its loops are unrolled less), which may change where the compiler
forms fused multiply-adds, so those results are compared to 1e-5, not bit for bit.
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


def rel(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / (den if den > 0 else 1.0))


def dev(x, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(x), dtype=dtype).cuda()


# (m, d, k): several kernel shapes in one batch, ragged sizes, a one-workgroup layer, both kernel families,
# and one layer (k=32, d=8) that only the stream path serves
MIXED = [(70_001, 1, 4), (513, 1, 4), (20_011, 2, 8), (33_333, 1, 4), (6_007, 4, 256), (9_999, 1, 4),
         (3_001, 2, 100), (2_050, 8, 32), (40_000, 2, 8), (257, 1, 4)]


def _mixed_layers(dist):
    out = []
    for i, (m, d, k) in enumerate(MIXED):
        W, C0, G = wl.random_problem(m, d, k, seed=700 + i, std=0.5, spread=1.5)
        C0 = C0 + 0.01 * np.random.default_rng(i).standard_normal(C0.shape)
        tau = 0.1 if dist == wl.DIST_L2 else 0.05
        out.append((W.astype(np.float32), C0.astype(np.float32), G.astype(np.float32), tau))
    return out


@pytest.mark.parametrize("dist", [wl.DIST_L2, wl.DIST_SQL2])
def test_mixed_batch_matches_oracle_and_single_calls(dist):
    layers = _mixed_layers(dist)
    n = len(layers)
    b = binding.Batch(n)
    Wd = [dev(L[0]) for L in layers]
    Cd = [dev(L[1]) for L in layers]
    Gd = [dev(L[2]) for L in layers]
    taus = [L[3] for L in layers]
    tol, iters = 1e-5, 30
    fw = b.forward(list(zip(Wd, Cd)), taus, tol, iters, dist, want_assign=True)
    assert 1 <= b.launches() <= 4          # four persistent kernel shapes in MIXED, one launch each
    bw = b.backward(Gd, binding.BWD_IMPLICIT, tol=1e-6, max_iter=60, alpha=1.0)
    jf = b.backward(Gd, binding.BWD_JFB)
    # explicit-Jacobian mode: the k=4, d=1 layers share one launch, the others are refused or solved in their turn
    dn = b.backward(Gd, binding.BWD_DENSE, strict=False)
    for i, (m, d, k) in enumerate(MIXED):
        if k * d <= 16 and k in (2, 4, 8, 16):
            assert dn[i]["status"] == 0 and dn[i]["info"].converged
            rd = orc.backward(layers[i][0], fw[i]["C"].cpu().numpy(), layers[i][3], dist, layers[i][2], mode="dense")
            assert rel(dn[i]["dW"].cpu().numpy(), rd["dW"]) < TOL_GRAD, i
            assert dn[i]["info"].path == (binding.PATH_PERSISTENT if (k, d) == (4, 1) else binding.PATH_STREAM)
        else:
            assert dn[i]["status"] == 6
    single = binding.Context(0)
    for i, (W, C0, G, tau) in enumerate(layers):
        ref = orc.soft_kmeans(W, C0, tau, tol, iters, dist)
        Cstar = fw[i]["C"].cpu().numpy()
        assert fw[i]["status"] == 0
        assert rel(Cstar, ref["C"]) < TOL_VAL, i
        assert abs(fw[i]["info"].iters - ref["iters"]) <= 1, i
        # E-step outputs and the backward against the oracle at the kernel's own C* (as in the per-layer tests:
        # this separates them from the solve, whose result is compared just above)
        assert rel(fw[i]["Wq"].cpu().numpy(), orc.soft_quantize(W, Cstar, tau, dist)) < TOL_VAL, i
        np.testing.assert_array_equal(fw[i]["assign"].cpu().numpy(), orc.hard_assign_f32(W, Cstar))
        rb = orc.backward(W, Cstar, tau, dist, G, mode="implicit", tol=1e-6, max_iter=60, alpha=1.0)
        assert rel(bw[i]["dW"].cpu().numpy(), rb["dW"]) < TOL_GRAD, i
        rj = orc.backward(W, Cstar, tau, dist, G, mode="jfb")
        assert rel(jf[i]["dW"].cpu().numpy(), rj["dW"]) < TOL_GRAD, i
        # the same layer through the per-layer entry points
        s = single.forward(Wd[i], Cd[i], tau, tol, iters, dist, want_assign=True)
        assert s["info"].path == fw[i]["info"].path
        assert abs(s["info"].iters - fw[i]["info"].iters) <= 1
        assert rel(fw[i]["C"].cpu().numpy(), s["C"].cpu().numpy()) < 1e-5
        assert rel(fw[i]["Wq"].cpu().numpy(), s["Wq"].cpu().numpy()) < 1e-5
        sb = single.backward(Gd[i], binding.BWD_IMPLICIT, tol=1e-6, max_iter=60, alpha=1.0)
        assert abs(sb["info"].iters - bw[i]["info"].iters) <= 1
        assert rel(bw[i]["dW"].cpu().numpy(), sb["dW"].cpu().numpy()) < 1e-4, i
    paths = [fw[i]["info"].path for i in range(n)]
    assert paths[7] == binding.PATH_STREAM and paths.count(binding.PATH_PERSISTENT) == n - 1
    single.close()
    b.close()


def test_batch_larger_than_one_launch_and_repeated_calls():
    # 24 layers of ~150k scalars: 147 workgroups each at 4 KiB of LDS; with 4 KiB tiles the device holds
    # several layers per launch but not all 24, so the batch must split, and a second call must reuse its state
    dist = wl.DIST_SQL2
    n = 24
    Ws, Cs = [], []
    for i in range(n):
        cfg = wl.sweep_config(5 + (i % 3), 4, dist)
        p = wl.make_problem(cfg, dist, m=150_000 + 1_001 * i)
        Ws.append(dev(p.W))
        Cs.append(dev(p.C0))
        tol0 = cfg.tol
    taus = [wl.sweep_config(5 + (i % 3), 4, dist).tau for i in range(n)]
    b = binding.Batch(n)
    first = b.forward(list(zip(Ws, Cs)), taus, tol0, 40, dist, want_Wq=False)
    launches = b.launches()
    assert launches >= 1
    again = b.forward(list(zip(Ws, Cs)), taus, tol0, 40, dist, want_Wq=False)
    assert b.launches() == launches
    for i in range(n):
        assert torch.equal(first[i]["C"], again[i]["C"])
        assert first[i]["info"].iters == again[i]["info"].iters
    for i in (0, 7, 23):
        W = Ws[i].cpu().numpy()
        ref = orc.soft_kmeans(W, Cs[i].cpu().numpy(), taus[i], tol0, 40, dist)
        assert rel(first[i]["C"].cpu().numpy(), ref["C"]) < TOL_VAL
        assert abs(first[i]["info"].iters - ref["iters"]) <= 1
    b.close()


def test_batch_reports_per_layer_failures_and_keeps_going():
    dist = wl.DIST_SQL2
    layers = []
    for i in range(3):
        W, C0, _ = wl.random_problem(5_000 + i, 1, 4, seed=900 + i, std=0.5, spread=1.5)
        layers.append((W.astype(np.float32), C0.astype(np.float32)))
    layers[1][0][17, 0] = np.nan      # the middle layer has a non-finite weight
    b = binding.Batch(3)
    out = b.forward([(dev(W), dev(C0)) for W, C0 in layers], 0.05, 1e-5, 20, dist, strict=False)
    assert [o["status"] for o in out] == [0, 4, 0]          # IDKM_ERR_NONFINITE for layer 1 only
    for i in (0, 2):
        ref = orc.soft_kmeans(layers[i][0], layers[i][1], 0.05, 1e-5, 20, dist)
        assert rel(out[i]["C"].cpu().numpy(), ref["C"]) < TOL_VAL
    with pytest.raises(binding.IdkmError):
        b.forward([(dev(W), dev(C0)) for W, C0 in layers], 0.05, 1e-5, 20, dist)
    # backward of a layer whose forward failed is refused, the others still run
    G = [dev(np.ones_like(W)) for W, _ in layers]
    bw = b.backward(G, binding.BWD_JFB, strict=False)
    assert [o["status"] for o in bw] == [0, 5, 0]           # IDKM_ERR_NO_FORWARD
    b.close()


def test_batch_argument_errors():
    lib = binding.load_library()
    import ctypes as C
    h = C.c_void_p()
    assert lib.idkm_batch_create(C.byref(h), 0, 0) == 1
    assert lib.idkm_batch_create(C.byref(h), 0, 5000) == 1
    b = binding.Batch(2)
    W, C0, _ = wl.random_problem(1000, 1, 4, seed=1)
    three = [(dev(W), dev(C0))] * 3
    with pytest.raises(binding.IdkmError):
        b.forward(three, 0.05, 1e-5, 5, wl.DIST_SQL2)       # more layers than contexts
    assert lib.idkm_batch_context(b._h, 2) is None
    assert lib.idkm_batch_context(b._h, 1) is not None
    b.close()
