"""Pins of the oracle's code packing (Sec. 3: b bits per sub-vector, k = 2^b) against things other than itself:
a hand-worked bit stream, Python big-integer arithmetic, and brute force for the closest-codeword map."""
import numpy as np
import pytest

from oracle import idkm_oracle as orc


def test_code_bits():
    assert [orc.code_bits(k) for k in (1, 2, 3, 4, 5, 16, 17, 256, 1000, 1024)] == [1, 1, 2, 2, 3, 4, 5, 8, 10, 10]


def test_hand_worked_stream():
    # k = 4 (2 bits): codes 1,2,3,0,3 -> bits (LSB first) 10 01 11 00 11 -> 0b11_00_11_10_01 = 0x339
    assert orc.pack_codes([1, 2, 3, 0, 3], 4).tolist() == [0x339]
    # k = 8 (3 bits), 11 codes of value 5 (101): 33 bits, so bit 32 spills into a second word
    w = orc.pack_codes([5] * 11, 8)
    stream = sum(5 << (3 * i) for i in range(11))
    assert w.tolist() == [stream & 0xFFFFFFFF, stream >> 32]
    # k = 2: one bit per code
    assert orc.pack_codes([1, 0, 0, 1, 1], 2).tolist() == [0b11001]


@pytest.mark.parametrize("k", [2, 3, 4, 16, 100, 256, 1024])
@pytest.mark.parametrize("m", [1, 31, 32, 33, 1000])
def test_against_big_integer_arithmetic_and_round_trip(k, m):
    rng = np.random.default_rng(k * 1000 + m)
    a = rng.integers(0, k, size=m)
    b = orc.code_bits(k)
    big = 0
    for i, c in enumerate(a.tolist()):
        big |= c << (i * b)
    nwords = (m * b + 31) // 32
    expect = [(big >> (32 * t)) & 0xFFFFFFFF for t in range(nwords)]
    words = orc.pack_codes(a, k)
    assert words.dtype == np.uint32 and words.tolist() == expect
    assert np.array_equal(orc.unpack_codes(words, m, k), a)


def test_hard_quantize_is_the_closest_codeword_by_brute_force():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((200, 3)).astype(np.float32)
    C = rng.standard_normal((7, 3)).astype(np.float32)
    Q = orc.hard_quantize(W, C)
    for i in range(200):
        dist = [float(np.sum((W[i].astype(np.float64) - C[j].astype(np.float64)) ** 2)) for j in range(7)]
        j = int(np.argmin(dist))
        assert np.array_equal(Q[i], C[j])
    asg = orc.hard_assign_f32(W, C)
    brute = sum(min(float(np.sum((W[i].astype(np.float64) - C[j].astype(np.float64)) ** 2)) for j in range(7)) for i in range(200))
    assert abs(orc.cluster_objective(W, C, asg) - brute) < 1e-9 * brute
