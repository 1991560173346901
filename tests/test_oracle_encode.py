"""Pins of the oracle's ANN code (quantise -> +-1 projection -> shift) against closed forms.

Sec. 5.1 only says: project to a shared low-dimensional random subspace, quantise to low bit
width (8 bit by default).  The integer pipeline is this build's reading; what is checked here
are hand-computed values that a wrong rounding, sign, transpose or shift would break.
"""
import numpy as np
import pytest

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32, make_codec


def enc(x, R, qscale, shift):
    return oracle.encode(np.asarray(x, np.float32), np.asarray(R, np.int8), qscale, shift)


def test_zero_vector_gives_zero_code():
    R = make_codec(0, 1, 64, 32).R
    assert not enc(np.zeros((3, 64)), R, 127 / 4.5, 4).any()


def test_unit_coordinate_reads_one_row_of_R():
    # x = 4.5 * e_t quantises to 127 * e_t, so y_j = 127 R[t][j] and c_j = floor((+-127 + 8) / 16) = +-8
    codec = make_codec(0, 1, 64, 32)
    for t in (0, 5, 63):
        x = np.zeros((1, 64), np.float32)
        x[0, t] = 4.5
        c = enc(x, codec.R, codec.qscale, codec.shift)[0]
        assert np.array_equal(c, 8 * codec.R[t].astype(np.int8))


def test_projection_uses_R_as_d_by_r_not_transposed():
    # R = [[1, 1], [1, -1], [1, 1]] (d=3, r=2), xq = (2, 4, 6): y = (12, 4); shift 1: c = floor((y+1)/2) = (6, 2)
    R = np.array([[1, 1], [1, -1], [1, 1]], np.int8)
    c = enc([[2.0, 4.0, 6.0]], R, 1.0, 1)[0]
    assert c.tolist() == [6, 2]


@pytest.mark.parametrize("x,xq", [(0.25, 0), (0.75, 2), (1.25, 2), (1.75, 4), (-0.25, 0), (-0.75, -2),
                                  (-1.25, -2), (0.3, 1), (-0.3, -1), (100.0, 127), (-100.0, -127)])
def test_quantiser_rounds_half_to_even_and_saturates(x, xq):
    # qscale = 2 makes x * qscale exact; d = 2 with R = [1, 1]^T and shift 1 gives c = floor((2 xq + 1)/2) = xq
    R = np.array([[1], [1]], np.int8)
    assert enc([[x, x]], R, 2.0, 1)[0, 0] == xq


@pytest.mark.parametrize("y,c", [(0, 0), (7, 0), (8, 1), (-8, 0), (-9, -1), (23, 1), (24, 2), (-24, -1), (-25, -2)])
def test_shift_is_floor_with_half_added(y, c):
    # d = 1, R = [[1]], qscale = 1: y = xq; shift 4: c = floor((y + 8) / 16)
    R = np.array([[1]], np.int8)
    assert enc([[float(y)]], R, 1.0, 4)[0, 0] == c


def test_code_saturates_at_127_never_minus_128():
    d = 128
    R = np.ones((d, 2), np.int8)
    R[:, 1] = -1
    c = enc(np.full((1, d), 4.5), R, 127 / 4.5, 4)[0]      # y = +-16256 -> +-1016 -> +-127
    assert c.tolist() == [127, -127]


def test_matches_vectorised_integer_pipeline():
    rng = np.random.default_rng(1)
    codec = make_codec(0, 2, 128, 32)
    x = (rng.standard_normal((500, 128)) * 1.1).astype(np.float32)
    xq = np.clip(np.rint(x * codec.qscale), -127, 127).astype(np.int64)     # float32 product, half-even
    y = xq @ codec.R.astype(np.int64)
    c = np.clip((y + 8) >> 4, -127, 127).astype(np.int8)
    assert np.array_equal(enc(x, codec.R, codec.qscale, codec.shift), c)


def test_antisymmetric_up_to_the_rounding_half():
    rng = np.random.default_rng(2)
    codec = make_codec(0, 2, 128, 32)
    x = rng.standard_normal((200, 128)).astype(np.float32)
    a = enc(x, codec.R, codec.qscale, codec.shift).astype(np.int32)
    b = enc(-x, codec.R, codec.qscale, codec.shift).astype(np.int32)
    s = a + b                                   # floor(u) + floor(-u + 1) in {0, 1}: 1 only at y + 8 = 0 mod 16
    assert s.min() >= 0 and s.max() <= 1 and (s == 0).mean() > 0.9


def test_bf16_storage_is_read_as_its_exact_value():
    rng = np.random.default_rng(3)
    codec = make_codec(0, 2, 128, 32)
    x = rng.standard_normal((64, 128)).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    assert np.array_equal(oracle.encode(bits, codec.R, codec.qscale, codec.shift),
                          enc(bf16_bits_to_f32(bits), codec.R, codec.qscale, codec.shift))


def test_scores_are_integers_below_2_pow_24():
    # what makes bit-exact decisions possible on any device: |c.c'| <= r * 127^2 and the L2 form
    # |2 c.c' - c'.c'| <= 3 r 127^2 both stay below 2^24 for r <= 64
    for r in (32, 64):
        assert 3 * r * 127 * 127 < 2 ** 24


# ------------------------------------------------------------------ codes of 2 and 4 bits per entry, packed
# (appendix, "Quantization precision for ANN matching": the bit width of the retrieval codes is varied)

def _np_unpack(packed, r, bits):
    per = 8 // bits
    j = np.arange(r)
    c = (packed[..., j // per].astype(np.int32) >> (bits * (j % per))) & ((1 << bits) - 1)
    return np.where(c >= 1 << (bits - 1), c - (1 << bits), c).astype(np.int8)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_packed_codes_are_the_8_bit_codes_saturated_to_the_narrow_range(bits, dtype):
    from workloads import make_codec, to_storage
    rng = np.random.default_rng(bits)
    d, r = 128, 32
    codec = make_codec(0, 1, d, r)
    x = to_storage((1.2 * rng.standard_normal((3, 50, d))).astype(np.float32), dtype)
    lim = (1 << (bits - 1)) - 1
    for shift in (4, 6, 8, 9):
        wide = oracle.encode(x, codec.R, codec.qscale, shift)
        packed = oracle.encode_packed(x, codec.R, codec.qscale, shift, bits)
        assert packed.shape == (3, 50, r * bits // 8) and packed.dtype == np.uint8
        got = _np_unpack(packed, r, bits)
        assert np.array_equal(got, np.clip(wide, -lim, lim))
        assert np.array_equal(oracle.unpack_codes(packed, r, bits), got)
        if bits == 8:
            assert np.array_equal(packed.view(np.int8), wide)
        elif shift == 4:
            assert (np.abs(got) == lim).any() and (np.abs(wide) > lim).any()      # the narrow range does saturate here


def test_packed_layout_by_hand():
    # d = 4, r = 4, R = identity-like signs: y = +-xq, shift 1: c = floor((y + 1) / 2)
    R = np.array([[1, 0, 0, 0], [0, 1, 0, 0], [0, 0, -1, 0], [0, 0, 0, 1]], np.int8)
    x = np.array([[2.0, -2.0, 9.0, 100.0]], np.float32)          # xq = 2, -2, 9, 100 -> y = 2, -2, -9, 100
    # c8 = floor(3/2), floor(-1/2), floor(-8/2), floor(101/2) = 1, -1, -4, 50
    assert oracle.encode(x, R, 1.0, 1).tolist() == [[1, -1, -4, 50]]
    # 4 bits: 1, -1, -4, 7 -> nibbles 0x1, 0xF, 0xC, 0x7 -> bytes 0xF1, 0x7C
    assert oracle.encode_packed(x, R, 1.0, 1, 4).tolist() == [[0xF1, 0x7C]]
    # 2 bits: 1, -1, -1, 1 -> 01, 11, 11, 01 from the low end -> 0b01111101
    assert oracle.encode_packed(x, R, 1.0, 1, 2).tolist() == [[0b01111101]]
    assert oracle.unpack_codes(np.array([[0xF1, 0x7C]], np.uint8), 4, 4).tolist() == [[1, -1, -4, 7]]
    assert oracle.unpack_codes(np.array([[0b01111101]], np.uint8), 4, 2).tolist() == [[1, -1, -1, 1]]
