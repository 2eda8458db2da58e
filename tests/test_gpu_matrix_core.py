"""The matrix-core kernels (d = 4, 17 <= k <= 256: the forward loop for both energies, the (dF/dC)^T passes for the
squared one; persistent and stream path) against the float64 oracle.

That loop evaluates the exponent of Eq. "aterms" in its expanded form  -s^2|w|^2 + 2 s^2 w.c - s^2|c|^2  (one
16 x 16 x 4 matrix product per tile) instead of summing squared differences, so these cases aim at what the expansion
could get wrong: codebooks that do not fill the last block of 16, tiles that end inside a 16-vector step, data far
from the origin (the three terms cancel; the plain norm takes a square root of the result), rows whose weights all
underflow before the row shift, and one-workgroup layers.  Bars as everywhere: C*, Wq 1e-4 norm-wise, hard assignments bit-exact on the kernel's own C*.
"""
import numpy as np
import pytest
import torch

from oracle import idkm_oracle as orc
from paper_2312_07759_amd import binding
from paper_2312_07759_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL_VAL = 1e-4
BOTH = pytest.mark.parametrize("dist", [wl.DIST_SQL2, wl.DIST_L2], ids=["sql2", "l2"])


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
    yield c
    c.close()


def _check(ctx, W, C0, tau, iters, tol=0.0, DIST=wl.DIST_SQL2, path=binding.PATH_PERSISTENT):
    W, C0 = W.astype(np.float32), C0.astype(np.float32)
    ctx.set_path(path)
    try:
        out = ctx.forward(dev(W), dev(C0), tau, tol, iters, DIST, want_assign=True)
    finally:
        ctx.set_path(binding.PATH_PERSISTENT)
    assert out["info"].path == path
    ref = orc.soft_kmeans(W, C0, tau, tol, iters, DIST)
    Cg = out["C"].cpu().numpy()
    assert np.isfinite(Cg).all()
    assert abs(out["info"].iters - ref["iters"]) <= (0 if tol == 0.0 else 1)
    assert rel(Cg, ref["C"]) < TOL_VAL, rel(Cg, ref["C"])
    assert rel(out["Wq"].cpu().numpy(), orc.soft_quantize(W, Cg, tau, DIST)) < TOL_VAL
    assert np.array_equal(out["assign"].cpu().numpy(), orc.hard_assign_f32(W, Cg))
    # without the assignment the evaluation at C* runs on the matrix cores as well (persistent path): same C*,
    # Wq to the same bar, and a backward after it sees the same n*, F*
    ctx.set_path(path)
    try:
        out2 = ctx.forward(dev(W), dev(C0), tau, tol, iters, DIST, want_assign=False)
    finally:
        ctx.set_path(binding.PATH_PERSISTENT)
    assert np.array_equal(out2["C"].cpu().numpy(), Cg) and out2["info"].iters == out["info"].iters
    assert rel(out2["Wq"].cpu().numpy(), orc.soft_quantize(W, Cg, tau, DIST)) < TOL_VAL
    return out, ref


# (m, k): every register variant (k <= 64, <= 128, <= 256), codebooks that end inside a block of 16, tiles that end
# inside a step, fewer vectors than one step, several workgroups with a ragged last one
@pytest.mark.parametrize("m,k", [(4_001, 17), (9_973, 33), (1_000, 64), (20_011, 100), (7_777, 128), (40_001, 130),
                                 (30_000, 255), (65_537, 256), (300, 256), (19, 17)])
@BOTH
def test_shapes(ctx, m, k, dist):
    W, C0, _ = wl.random_problem(m, 4, k, seed=1000 + m % 97 + k, std=0.5, spread=1.5)
    C0 = C0 + 0.01 * np.random.default_rng(k).standard_normal(C0.shape)
    _check(ctx, W, C0, 0.3, 20, DIST=dist)


@BOTH
def test_data_far_from_the_origin(ctx, dist):
    # |w| is 100 times the spread of the data: without a reference point inside the data the expanded exponent
    # loses about four digits here
    rng = np.random.default_rng(5)
    m, k = 30_011, 64
    W = 5.0 + 0.05 * rng.standard_normal((m, 4))
    C0 = W[rng.choice(m, k, replace=False)] + 0.002 * rng.standard_normal((k, 4))
    _check(ctx, W, C0, 1e-3 if dist == wl.DIST_SQL2 else 1e-2, 25, DIST=dist)


@pytest.mark.parametrize("tau", [2e-4, 2e-3])
def test_rows_that_underflow_before_the_shift(ctx, tau):
    # a few vectors lie hundreds of kernel widths from every codeword: their unshifted weights are all zero in
    # float32, and the row is redone with the shift by its maximum.  At the smaller temperature the codewords lie
    # more than 100 squared kernel widths from their mean and the loop adds their norms to the exponent; at the
    # larger one it folds them into factors instead, and the redone row has to stay within range there too.
    rng = np.random.default_rng(6)
    m, k = 12_345, 100
    W = 0.05 * rng.standard_normal((m, 4))
    far = rng.choice(m, 40, replace=False)
    W[far] += rng.choice([-1.0, 1.0], size=(40, 4)) * 1.5
    C0 = W[rng.choice(np.setdiff1d(np.arange(m), far), k, replace=False)].copy()
    spread = ((C0 - C0.mean(0)) ** 2).sum(1).max() * np.log2(np.e) / tau
    assert spread > 150 if tau < 1e-3 else spread < 60
    e = ((W[far, None, :] - C0[None, :, :]) ** 2).sum(-1).min(1)
    assert (e / tau * np.log2(np.e) > 200).all()          # beyond float32's exponent range without the shift
    _check(ctx, W, C0, tau, 15)


@BOTH
def test_stops_like_the_oracle(ctx, dist):
    W, C0, _ = wl.random_problem(25_000, 4, 48, seed=77, std=0.5, spread=1.5)
    out, ref = _check(ctx, W, C0, 0.05 if dist == wl.DIST_SQL2 else 0.2, 200, tol=1e-5, DIST=dist)
    assert out["info"].converged == ref["converged"]


def test_codewords_on_top_of_vectors(ctx):
    # plain norm, initial codewords that ARE rows of W: the expanded squared distance of such a pair is zero only
    # up to rounding (possibly negative) before its square root is taken
    rng = np.random.default_rng(9)
    m, k = 20_000, 96
    W = 0.05 * rng.standard_normal((m, 4))
    C0 = W[rng.choice(m, k, replace=False)].copy()
    _check(ctx, W, C0, 5e-3, 12, DIST=wl.DIST_L2)


@BOTH
@pytest.mark.parametrize("path", [binding.PATH_PERSISTENT, binding.PATH_STREAM], ids=["persistent", "stream"])
def test_matches_the_vector_alu_kernels(ctx, dist, path):
    # the same solve with the matrix-core kernels switched off (vector ALU, summed squared differences)
    W, C0, G = wl.random_problem(50_021, 4, 200, seed=78, std=0.5, spread=1.5)
    W, C0, G = W.astype(np.float32), C0.astype(np.float32), G.astype(np.float32)
    ctx.set_path(path)
    try:
        a = ctx.forward(dev(W), dev(C0), 0.2, 0.0, 30, dist)
        ga = ctx.backward(dev(G), binding.BWD_IMPLICIT, tol=0.0, max_iter=10, alpha=1.0)
        ctx.set_matrix_cores(False)
        b = ctx.forward(dev(W), dev(C0), 0.2, 0.0, 30, dist)
        gb = ctx.backward(dev(G), binding.BWD_IMPLICIT, tol=0.0, max_iter=10, alpha=1.0)
    finally:
        ctx.set_matrix_cores(True)
        ctx.set_path(binding.PATH_PERSISTENT)
    assert a["info"].path == path and b["info"].path == path
    assert rel(a["C"].cpu().numpy(), b["C"].cpu().numpy()) < 2e-5
    # the two backward solves start from slightly different C*: a loose bar, the oracle comparisons are the test
    assert rel(ga["dW"].cpu().numpy(), gb["dW"].cpu().numpy()) < 2e-3


@BOTH
@pytest.mark.parametrize("m,k", [(4_001, 17), (20_011, 100), (65_537, 256), (300, 256), (19, 17), (700_001, 64)])
def test_stream_path_shapes(ctx, m, k, dist):
    # one launch per pass: chunks of up to 2304 vectors, a ragged last workgroup, more workgroups than compute units
    W, C0, _ = wl.random_problem(m, 4, k, seed=3000 + m % 97 + k, std=0.5, spread=1.5)
    C0 = C0 + 0.01 * np.random.default_rng(k).standard_normal(C0.shape)
    _check(ctx, W, C0, 0.3, 12 if m > 100_000 else 20, DIST=dist, path=binding.PATH_STREAM)


# ---- the (dF/dC)^T passes of the implicit backward on the matrix cores

TOL_GRAD = 1e-3


def _check_backward(ctx, W, C0, G, tau, iters=15, passes=12, alpha=1.0, path=binding.PATH_PERSISTENT, dist=wl.DIST_SQL2):
    W, C0, G = W.astype(np.float32), C0.astype(np.float32), G.astype(np.float32)
    ctx.set_path(path)
    try:
        out = ctx.forward(dev(W), dev(C0), tau, 0.0, iters, dist)
        Cg = out["C"].cpu().numpy()
        bi = ctx.backward(dev(G), binding.BWD_IMPLICIT, tol=0.0, max_iter=passes, alpha=alpha)
        bj = ctx.backward(dev(G), binding.BWD_JFB)
    finally:
        ctx.set_path(binding.PATH_PERSISTENT)
    assert bi["info"].path == path
    ri = orc.backward(W, Cg, tau, dist, G, "implicit", tol=0.0, max_iter=passes, alpha=alpha)
    if not (bi["info"].converged or ri["converged"]):
        assert bi["info"].iters == ri["iters"] and bi["info"].alpha == ri["alpha"]
    err = rel(bi["dW"].cpu().numpy(), ri["dW"])
    assert err < TOL_GRAD, err
    # the one-step variant: first and last pass only (on the matrix cores too for the squared energy, persistent path)
    assert rel(bj["dW"].cpu().numpy(), orc.backward(W, Cg, tau, dist, G, "jfb")["dW"]) < TOL_GRAD


@BOTH
@pytest.mark.parametrize("m,k", [(4_001, 17), (20_011, 100), (7_777, 128), (30_000, 255), (65_537, 256), (300, 256)])
def test_backward_shapes(ctx, m, k, dist):
    W, C0, G = wl.random_problem(m, 4, k, seed=2000 + m % 89 + k, std=0.5, spread=1.5)
    C0 = C0 + 0.01 * np.random.default_rng(k).standard_normal(C0.shape)
    _check_backward(ctx, W, C0, G, 0.3, dist=dist)


@BOTH
@pytest.mark.parametrize("m,k", [(4_001, 17), (20_011, 100), (65_537, 256), (300, 256)])
def test_backward_stream_path(ctx, m, k, dist):
    W, C0, G = wl.random_problem(m, 4, k, seed=2200 + m % 89 + k, std=0.5, spread=1.5)
    C0 = C0 + 0.01 * np.random.default_rng(k).standard_normal(C0.shape)
    _check_backward(ctx, W, C0, G, 0.3, path=binding.PATH_STREAM, dist=dist)


@BOTH
def test_backward_damped(ctx, dist):
    W, C0, G = wl.random_problem(15_000, 4, 64, seed=2100, std=0.5, spread=1.5)
    _check_backward(ctx, W, C0, G, 0.3, alpha=0.25, dist=dist)


@BOTH
def test_backward_data_far_from_the_origin(ctx, dist):
    rng = np.random.default_rng(15)
    m, k = 30_011, 64
    W = 5.0 + 0.05 * rng.standard_normal((m, 4))
    C0 = W[rng.choice(m, k, replace=False)] + 0.002 * rng.standard_normal((k, 4))
    G = rng.standard_normal((m, 4))
    _check_backward(ctx, W, C0, G, 1e-3 if dist == wl.DIST_SQL2 else 1e-2, iters=25, dist=dist)


def test_backward_codewords_on_top_of_vectors(ctx):
    # plain norm: the derivative of the energy is the unit vector (w - c)/|w - c|, zero where the two coincide; with
    # initial codewords that are rows of W and a single evaluation of F such pairs stay close to coincident
    rng = np.random.default_rng(19)
    m, k = 20_000, 96
    W = 0.05 * rng.standard_normal((m, 4))
    C0 = W[rng.choice(m, k, replace=False)].copy()
    G = rng.standard_normal((m, 4))
    _check_backward(ctx, W, C0, G, 5e-3, iters=1, passes=6, dist=wl.DIST_L2)


@pytest.mark.parametrize("tau", [2e-4, 2e-3])
def test_backward_rows_that_underflow(ctx, tau):
    rng = np.random.default_rng(16)
    m, k = 12_345, 100
    W = 0.05 * rng.standard_normal((m, 4))
    far = rng.choice(m, 40, replace=False)
    W[far] += rng.choice([-1.0, 1.0], size=(40, 4)) * 1.5
    C0 = W[rng.choice(np.setdiff1d(np.arange(m), far), k, replace=False)].copy()
    G = rng.standard_normal((m, 4))
    _check_backward(ctx, W, C0, G, tau, iters=15, passes=8)
