"""Pins for the oracle's quantizer, packing and dequantisation (CPU only).

The paper fixes only "weight-only, group size 128, 4/3 bit" (Sec. 4.1); these tests pin the
round-to-nearest reading against things that do not depend on the oracle's own formula:
a brute-force search over all 16 codes, closed-form lattices, and hand-written words."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import qtale_oracle as orc


def _rand_w(N, K, seed, std=0.02):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, K)) * std).astype(np.float32)


@pytest.mark.parametrize("bits", [4, 3, 2])
@pytest.mark.parametrize("N,K,G", [(8, 128, 128), (5, 688, 32), (7, 256, 32), (3, 40, 16), (4, 130, 128)])
def test_codes_are_the_nearest_representable_value(N, K, G, bits):
    W = _rand_w(N, K, seed=N * 1000 + K)
    codes, s, z = orc.quantize_rtn(W, bits, G)
    top = (1 << bits) - 1
    assert codes.min() >= 0 and codes.max() <= top
    assert z.min() >= 0 and z.max() <= top and np.all(z == np.rint(z))
    for n in range(N):
        for k in range(K):
            g = k // G
            sf, zz = float(s[n, g]), float(z[n, g])
            cand = [(c - zz) * sf for c in range(top + 1)]       # every representable value, fp64
            err = [abs(float(W[n, k]) - v) for v in cand]
            best = min(err)
            assert err[int(codes[n, k])] <= best + 1e-6 * sf, (n, k)


def test_error_bound_half_step():
    W = _rand_w(16, 512, seed=1)
    codes, s, z = orc.quantize_rtn(W, 4, 128)
    Wd = orc.dequantize(codes, s, z, 128)
    step = s.astype(np.float64)[:, np.arange(512) // 128]
    # zero-point rounding can push the grid by up to half a step at the far end of the range
    assert np.all(np.abs(W - Wd) <= step * (1.0 + 1e-3))
    inside = (codes > 0) & (codes < 15)
    assert np.all(np.abs(W - Wd)[inside] <= 0.5 * step[inside] * (1 + 1e-3))


def test_exact_lattice_is_reproduced():
    # weights that already are (j - z0) * s with an fp16-representable s reproduce exactly
    s0 = float(np.float16(0.0123))
    z0 = 6
    K = 64
    rng = np.random.default_rng(3)
    j = rng.integers(0, 16, size=(4, K))
    j[:, 0], j[:, 1] = 0, 15                                     # make the range span all codes
    W = ((j - z0) * s0).astype(np.float32)
    codes, s, z = orc.quantize_rtn(W, 4, K)
    assert np.all(z == z0)
    assert np.all(codes == j)
    np.testing.assert_allclose(orc.dequantize(codes, s, z, K), (j - z0) * float(s[0, 0]), rtol=0, atol=0)


def test_constant_zero_group_and_one_sided_groups():
    W = np.zeros((2, 32), dtype=np.float32)
    codes, s, z = orc.quantize_rtn(W, 4, 16)
    assert np.all(s == 1.0) and np.all(codes == z[:, [0]]) and np.all(orc.dequantize(codes, s, z, 16) == 0)
    Wp = np.abs(_rand_w(3, 32, 5)) + 0.01                        # all positive: range starts at 0
    codes, s, z = orc.quantize_rtn(Wp, 4, 32)
    assert np.all(z == 0) and codes.max() == 15
    codes, s, z = orc.quantize_rtn(-Wp, 4, 32)                   # all negative: range ends at 0
    assert np.all(z == 15) and codes.min() == 0


def test_requantizing_dequantized_weights_is_idempotent():
    W = _rand_w(6, 256, seed=9)
    codes, s, z = orc.quantize_rtn(W, 4, 32)
    Wd = orc.dequantize(codes, s, z, 32).astype(np.float32)
    codes2, s2, z2 = orc.quantize_rtn(Wd, 4, 32)
    # a group whose extreme codes are not both used can shrink its range; where the range is
    # unchanged the codes must be identical
    same = (s2 == s) & (z2 == z)
    assert same.mean() > 0.5
    g = np.arange(256) // 32
    assert np.all((codes2 == codes)[same[:, g]])


def test_three_bit_range():
    W = _rand_w(4, 128, seed=11)
    codes, s, z = orc.quantize_rtn(W, 3, 128)
    assert codes.max() <= 7 and z.max() <= 7
    Wd = orc.dequantize(codes, s, z, 128)
    assert np.max(np.abs(W - Wd)) <= float(s.max()) * 1.001


def test_pack_layout_hand_written_words():
    codes = np.array([[0, 1, 2, 3, 4, 5, 6, 7, 15, 0, 0, 0, 0, 0, 0, 8, 9, 10]], dtype=np.uint8)
    words = orc.pack_codes(codes)
    assert words.dtype == np.uint32 and words.shape == (1, 3)
    assert words[0, 0] == 0x76543210
    assert words[0, 1] == 0x8000000F
    assert words[0, 2] == 0x000000A9                              # tail padded with code 0
    assert np.array_equal(orc.unpack_codes(words, 18), codes)


def test_three_bit_pack_hand_written_words():
    # bit stream, least-significant first: code k sits at bits 3k..3k+2 of its row
    codes = np.array([[1, 2, 3]], dtype=np.uint8)
    words = orc.pack_codes(codes, 3)
    assert words.dtype == np.uint32 and words.shape == (1, 3)    # one 32-code block = 3 words
    assert list(words[0]) == [1 + (2 << 3) + (3 << 6), 0, 0]
    # codes 10 and 21 straddle the word boundaries (bits 30-32 and 63-65)
    codes = np.zeros((1, 32), dtype=np.uint8)
    codes[0, 10], codes[0, 21], codes[0, 31] = 0b110, 0b101, 0b111
    words = orc.pack_codes(codes, 3)
    assert list(words[0]) == [0b10 << 30, 0b1 | (0b1 << 31), 0b10 | (0b111 << 29)]
    assert np.array_equal(orc.unpack_codes(words, 32, 3), codes)


def test_three_bit_pack_matches_big_integer_bit_stream():
    rng = np.random.default_rng(4)
    for K in (32, 40, 688, 96):
        codes = rng.integers(0, 8, size=(3, K)).astype(np.uint8)
        words = orc.pack_codes(codes, 3)
        assert words.shape == (3, 3 * ((K + 31) // 32))
        for n in range(3):
            stream = 0
            for k in range(K):
                stream |= int(codes[n, k]) << (3 * k)            # arbitrary-precision integer
            want = [(stream >> (32 * w)) & 0xFFFFFFFF for w in range(words.shape[1])]
            assert [int(v) for v in words[n]] == want
        assert np.array_equal(orc.unpack_codes(words, K, 3), codes)


def test_three_bit_lattice_and_one_sided_groups():
    s0 = float(np.float16(0.031))
    j = np.array([[0, 7, 3, 5, 1, 6, 2, 4]] * 2)
    W = ((j - 3) * s0).astype(np.float32)
    codes, s, z = orc.quantize_rtn(W, 3, 8)
    assert np.all(z == 3) and np.all(codes == j)
    Wp = np.abs(_rand_w(3, 32, 5)) + 0.01
    codes, s, z = orc.quantize_rtn(Wp, 3, 32)
    assert np.all(z == 0) and codes.max() == 7
    codes, s, z = orc.quantize_rtn(-Wp, 3, 32)
    assert np.all(z == 7) and codes.min() == 0


def test_two_bit_pack_hand_written_words():
    codes = np.array([[3, 0, 1, 2] + [0] * 11 + [3, 2, 1]], dtype=np.uint8)       # K = 18: two words
    words = orc.pack_codes(codes, 2)
    assert words.dtype == np.uint32 and words.shape == (1, 2)
    assert words[0, 0] == (3 | (1 << 4) | (2 << 6) | (3 << 30))
    assert words[0, 1] == (2 | (1 << 2))
    assert np.array_equal(orc.unpack_codes(words, 18, 2), codes)
    rng = np.random.default_rng(8)
    codes = rng.integers(0, 4, size=(4, 688)).astype(np.uint8)
    assert np.array_equal(orc.unpack_codes(orc.pack_codes(codes, 2), 688, 2), codes)


def test_two_bit_lattice():
    s0 = float(np.float16(0.07))
    j = np.array([[0, 3, 1, 2, 2, 1, 3, 0]] * 2)
    W = ((j - 1) * s0).astype(np.float32)
    codes, s, z = orc.quantize_rtn(W, 2, 8)
    assert np.all(z == 1) and np.all(codes == j)


def test_pack_roundtrip_ragged():
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 16, size=(5, 688)).astype(np.uint8)
    assert np.array_equal(orc.unpack_codes(orc.pack_codes(codes), 688), codes)


def test_ragged_last_group_uses_only_its_members():
    # K = 688 with G = 32 leaves a last group of 16; make those 16 tiny so their scale must be tiny
    W = _rand_w(2, 688, seed=21)
    W[:, 672:] *= 1e-2
    codes, s, z = orc.quantize_rtn(W, 4, 32)
    assert s.shape == (2, 22)
    assert np.all(s[:, 21].astype(np.float64) < 0.1 * s[:, :21].astype(np.float64).min())
    Wd = orc.dequantize(codes, s, z, 32)
    assert np.max(np.abs(W - Wd)[:, 672:]) <= float(s[:, 21].max()) * 1.001


def test_dequant_closed_form():
    codes = np.array([[0, 15, 7, 8]], dtype=np.uint8)
    s = np.array([[0.5, 0.25]], dtype=np.float16)
    z = np.array([[7.0, 8.0]], dtype=np.float16)
    np.testing.assert_array_equal(orc.dequantize(codes, s, z, 2), [[-3.5, 4.0, -0.25, 0.0]])


def test_packed_size_matches_shape_arithmetic():
    # LLaMA-7B-shaped layer: 4 bit codes + fp16 scale and zero per 128 weights
    P = si.C2.params_per_layer()
    assert P == 202375168
    assert P // 2 + 2 * 2 * (P // 128) == 101187584 + 6324224


def test_zero_point_is_never_negative_zero():
    W = np.abs(_rand_w(4, 64, 33)) + 0.01                        # lo = 0 -> -lo/s = -0.0
    _, _, z = orc.quantize_rtn(W, 4, 32)
    assert np.all(z.view(np.uint16) == 0)
