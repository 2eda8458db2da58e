"""Packed b-bit codes and the reconstruction q(W, C) (Sec. 3) on the GPU against the oracle: integer and byte work,
so every comparison is bit-exact."""
import numpy as np
import pytest
import torch

from oracle import idkm_oracle as orc
from paper_2312_07759_amd import binding
from paper_2312_07759_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def words_u32(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("k", [2, 3, 4, 16, 100, 256, 1024])
@pytest.mark.parametrize("m", [1, 31, 32, 33, 8191, 8192, 70_001])
def test_pack_matches_oracle_bit_for_bit(ctx, m, k):
    a = np.random.default_rng(m * 31 + k).integers(0, k, size=m).astype(np.int32)
    w = ctx.pack_codes(torch.from_numpy(a).cuda(), k)
    ref = orc.pack_codes(a, k)
    assert w.shape[0] == ref.shape[0] == binding.code_words(m, k)
    assert np.array_equal(words_u32(w), ref)
    assert binding.code_bits(k) == orc.code_bits(k)


@pytest.mark.parametrize("m,d,k", [(70_001, 1, 4), (20_011, 2, 8), (6_007, 4, 256), (3_001, 2, 100), (2_100, 4, 1024),
                                   (1_100, 8, 512), (5, 1, 2)])
def test_forward_assign_pack_unpack_round_trip(ctx, m, d, k):
    W, C0, _ = wl.random_problem(m, d, k, seed=m + k, std=0.5, spread=1.5)
    W = W.astype(np.float32)
    out = ctx.forward(torch.from_numpy(W).cuda(), torch.from_numpy(C0.astype(np.float32)).cuda(), 0.05, 1e-5, 10,
                      wl.DIST_SQL2, want_assign=True)
    Cg = out["C"].cpu().numpy()
    asg = out["assign"]
    assert np.array_equal(asg.cpu().numpy(), orc.hard_assign_f32(W, Cg))
    words = ctx.pack_codes(asg, k)
    assert np.array_equal(words_u32(words), orc.pack_codes(asg.cpu().numpy(), k))
    Wh = ctx.unpack_quantize(words, m, out["C"]).cpu().numpy()
    ref = orc.hard_quantize(W, Cg)
    assert np.array_equal(Wh.view(np.uint32), ref.view(np.uint32))          # bitwise copies of codebook rows
    assert np.array_equal(orc.unpack_codes(words_u32(words), m, k), asg.cpu().numpy())


def test_full_size_stream_of_the_headline_tensor(ctx):
    p = wl.make_problem("C3", wl.DIST_SQL2)
    out = ctx.forward(torch.from_numpy(p.W).cuda(), torch.from_numpy(p.C0).cuda(), p.tau, p.tol, p.max_iter, wl.DIST_SQL2,
                      want_assign=True, want_Wq=False)
    words = ctx.pack_codes(out["assign"], p.cfg.k)
    assert words.shape[0] * 4 == p.cfg.m * 2 // 8                              # 2 bits per weight
    a = out["assign"].cpu().numpy()
    assert np.array_equal(words_u32(words), orc.pack_codes(a, p.cfg.k))
    Wh = ctx.unpack_quantize(words, p.cfg.m, out["C"]).cpu().numpy()
    assert np.array_equal(Wh, out["C"].cpu().numpy()[a])


def test_invalid_code_gives_nan_and_argument_errors(ctx):
    # k = 3 uses 2 bits; the value 3 cannot come from pack_codes of valid assignments
    words = torch.tensor([0b11_10_01_00], dtype=torch.int32).cuda()
    Cb = torch.tensor([[1.0], [2.0], [3.0]]).cuda()
    Wh = ctx.unpack_quantize(words, 4, Cb).cpu().numpy()
    assert Wh[:3, 0].tolist() == [1.0, 2.0, 3.0] and np.isnan(Wh[3, 0])
    lib = binding.load_library()
    assert lib.idkm_code_words(10, 0) == -1 and lib.idkm_code_words(10, 2000) == -1
    with pytest.raises(binding.IdkmError):
        ctx.pack_codes(torch.zeros(4, dtype=torch.int32).cuda(), 2000)
    assert ctx.pack_codes(torch.zeros(0, dtype=torch.int32).cuda(), 4).shape[0] == 0
