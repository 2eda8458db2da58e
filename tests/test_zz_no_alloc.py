"""idkm_forward_noalloc (the entry point for callers that cannot allocate) against idkm_forward, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input: the array in the library's device image keeps
the first call's contents, and nothing of them may leak into the second result.  Both entry points run the same
kernels in the same launch configuration, so the results are compared bit for bit (which is inside every tolerance of
the parity tests); a third call checks the size limit.
"""
import numpy as np
import pytest
import torch

from paper_2312_07759_amd import binding
from paper_2312_07759_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _both(ctx, p, dist, want_A):
    W, C0 = _dev(p.W), _dev(p.C0)
    m, d = p.W.shape
    k = p.C0.shape[0]
    ref = ctx.forward(W, C0, p.tau, p.tol, p.max_iter, dist, want_A=want_A, want_Wq=True, want_assign=True)
    out = dict(C=torch.full((k, d), float("nan"), device="cuda"), Wq=torch.full((m, d), float("nan"), device="cuda"),
               assign=torch.full((m,), -1, dtype=torch.int32, device="cuda"))
    if want_A:
        out["A"] = torch.full((m, k), float("nan"), device="cuda")
    info = binding.forward_noalloc(W, C0, p.tau, p.tol, p.max_iter, dist, out)
    assert ref["info"].path == binding.PATH_PERSISTENT and info.path == binding.PATH_PERSISTENT
    assert info.iters == ref["info"].iters and info.converged == ref["info"].converged
    assert info.residual == ref["info"].residual and info.empty_clusters == ref["info"].empty_clusters
    assert torch.equal(out["C"], ref["C"])
    assert torch.equal(out["Wq"], ref["Wq"])
    assert torch.equal(out["assign"], ref["assign"])
    if want_A:
        assert torch.equal(out["A"], ref["A"])
    return info


def test_no_alloc_forward_matches_the_context_entry_point_on_two_calls_in_a_row():
    ctx = binding.Context(0)
    try:
        dist = wl.DIST_SQL2
        big = wl.make_problem("C3", dist, m=300_007)        # 256 workgroups, ragged tail
        i1 = _both(ctx, big, dist, want_A=False)
        small = wl.make_problem("C2", wl.DIST_L2, m=20_011)  # fewer workgroups, k = 16, the other energy
        i2 = _both(ctx, small, wl.DIST_L2, want_A=True)
        assert i1.iters > 1 and i2.iters > 1
        # enqueue only (info = NULL), then read the outputs after a stream wait
        W, C0 = _dev(small.W), _dev(small.C0)
        out = dict(C=torch.zeros((16, 1), device="cuda"), Wq=torch.zeros((20_011, 1), device="cuda"))
        assert binding.forward_noalloc(W, C0, small.tau, small.tol, small.max_iter, wl.DIST_L2, out, want_info=False) is None
        torch.cuda.synchronize()
        ref = ctx.forward(W, C0, small.tau, small.tol, small.max_iter, wl.DIST_L2)
        assert torch.equal(out["C"], ref["C"]) and torch.equal(out["Wq"], ref["Wq"])
    finally:
        ctx.close()


def test_no_alloc_forward_rejects_what_it_cannot_hold():
    W = torch.zeros((1000, 1), device="cuda")
    out = dict(C=torch.zeros((3, 1), device="cuda"))
    with pytest.raises(binding.IdkmError) as e:      # k = 3 belongs to the other kernel family
        binding.forward_noalloc(W, torch.zeros((3, 1), device="cuda"), 0.1, 1e-6, 5, 1, out)
    assert e.value.status == 6
    big = torch.empty((9_400_001, 1), device="cuda")
    with pytest.raises(binding.IdkmError) as e:      # one weight beyond the stated maximum
        binding.forward_noalloc(big, torch.zeros((4, 1), device="cuda"), 0.1, 1e-6, 5, 1,
                                dict(C=torch.zeros((4, 1), device="cuda")))
    assert e.value.status == 6 and "9400000" in e.value.detail
