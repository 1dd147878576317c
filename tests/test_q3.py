"""3-bit weight format: pins of the CPU reference (hand-derived words, an independent packer, the pinned 4-bit reference
through an exact embedding, a closed form) and, on the GPU, parity of relax_unpack_q3 / relax_dequant_matmul_q3."""
import os

import numpy as np
import pytest

import oracle
from oracle import q3
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "q3_words.txt")


def golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                left, right = line.split("=>")
                pos, code = (int(v) for v in left.split())
                cases.append((pos, code, [int(w, 16) for w in right.split()]))
    return cases


@pytest.mark.parametrize("pos,code,words", golden_cases())
def test_hand_derived_words(pos, code, words):
    q = np.array([words], dtype=np.uint32)
    want = np.full((1, 32), -4, dtype=np.int8)
    want[0, pos] = code - 4
    assert np.array_equal(q3.unpack_q3(q, 1, 32), want)
    codes = np.zeros((1, 32), dtype=np.uint8)
    codes[0, pos] = code
    assert np.array_equal(wl.pack_codes3(codes), q)            # the generator's packer agrees with the same hand-derived words


def test_unpack_inverts_the_independent_packer():
    r = np.random.RandomState(5)
    codes = r.randint(0, 8, size=(7, 160)).astype(np.uint8)
    assert np.array_equal(q3.unpack_q3(wl.pack_codes3(codes), 7, 160), codes.astype(np.int8) - 4)


def test_matmul_equals_the_4bit_reference_on_embedded_codes():
    # u3 - 4 == (u3 + 4) - 8: the same matrix written as 4-bit codes must give the pinned 4-bit reference's product
    m, k, n = 9, 96, 3
    r = np.random.RandomState(6)
    codes = r.randint(0, 8, size=(m, k)).astype(np.uint8)
    s = (r.rand(m, k // 32) * 0.02 + 0.001).astype(np.float16).view(np.uint16)
    x = r.randn(n, k).astype(np.float32)
    ref4 = oracle.dequant_matmul(x, wl.pack_codes(codes + 4), s, m, k)
    got = q3.dequant_matmul_q3(x, wl.pack_codes3(codes), s, m, k)
    assert np.abs(got - ref4).max() <= 1e-5 * max(1.0, np.abs(ref4).max())
    assert np.array_equal(q3.dequantize_q3(wl.pack_codes3(codes), s, m, k).astype(np.float32), oracle.dequantize(wl.pack_codes(codes + 4), s, m, k))


def test_closed_form():
    m, k = 4, 64
    q = wl.pack_codes3(np.full((m, k), 7, dtype=np.uint8))                 # every weight 3 * 0.5
    s = np.full((m, k // 32), np.float16(0.5)).view(np.uint16)
    assert np.array_equal(q3.dequant_matmul_q3(np.ones((2, k), np.float32), q, s, m, k), np.full((2, m), 1.5 * k))


def test_quantiser_stays_in_range_and_close():
    w = wl.rng(3, 1).standard_normal((5, 64), dtype=np.float32) * np.float32(0.02)
    q, s = wl.quantize_q3(w)
    codes = q3.unpack_q3(q, 5, 64)
    assert codes.min() >= -3 and codes.max() <= 3
    step = np.repeat(s.view(np.float16).astype(np.float64), 32, axis=1)
    assert np.all(np.abs(q3.dequantize_q3(q, s, 5, 64) - w) <= 0.5 * step + 1e-6)
