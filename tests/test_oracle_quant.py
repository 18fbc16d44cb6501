"""Pins of the E4M3 encoder / decoder and the block quantiser of the oracle (CPU only).

The expected codes below follow from the OCP 8-bit floating point specification (E4M3: bias 7,
3 mantissa bits, subnormal step 2^-9, largest finite value 448 = 0x7E, 0x7F = NaN), worked out by
hand; none of them comes from a GPU run.
"""
import numpy as np
import pytest

from oracle import quant


def test_decode_known_codes():
    codes = np.array([0x00, 0x01, 0x07, 0x08, 0x38, 0x40, 0x44, 0x7E, 0x80, 0xB8, 0xFE], dtype=np.uint8)
    want = [0.0, 2.0 ** -9, 7 * 2.0 ** -9, 2.0 ** -6, 1.0, 2.0, 3.0, 448.0, -0.0, -1.0, -448.0]
    got = quant.e4m3_decode(codes)
    assert np.array_equal(got, np.array(want))
    assert np.signbit(got[8])
    assert np.isnan(quant.e4m3_decode(np.array([0x7F, 0xFF], dtype=np.uint8))).all()


def test_every_finite_code_survives_a_round_trip():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(quant.e4m3_encode(quant.e4m3_decode(codes)), codes)


def test_decode_is_monotonic_in_the_code():
    vals = quant.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    assert np.all(np.diff(vals) > 0)


@pytest.mark.parametrize("value, code", [
    (1.0, 0x38), (2.0, 0x40), (448.0, 0x7E), (2.0 ** -6, 0x08), (2.0 ** -9, 0x01),
    (2.0 ** -10, 0x00),      # tie between 0 and the smallest subnormal: even is 0
    (3 * 2.0 ** -10, 0x02),  # tie between 1 and 2 subnormal steps: even is 2
    (17.0, 0x58),            # tie between 16 (mantissa 000) and 18 (001): even is 16
    (19.0, 0x5A),            # tie between 18 (001) and 20 (010): even is 20
    (1.0625, 0x38), (1.1875, 0x3A),
    (15.5, 0x58),            # rounds up across the binade: 15 -> 16
    (463.9, 0x7E), (-3.0, 0xC4), (0.3, 0x2A),   # 0.3 = 1.2 * 2^-2 -> mantissa 1.25 (010)
])
def test_encode_rounds_to_nearest_even(value, code):
    assert int(quant.e4m3_encode(np.array([value]))[0]) == code


def test_encode_is_the_nearest_code_brute_force():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.uniform(-448, 448, 2000), rng.normal(0, 1, 2000), rng.normal(0, 0.01, 2000)])
    grid = quant.e4m3_decode(np.array([c for c in range(0x7F)], dtype=np.uint8))     # non-negative values, ascending
    got = quant.e4m3_decode(quant.e4m3_encode(x))
    nearest = np.abs(np.abs(x)[:, None] - grid[None, :]).min(axis=1)
    assert np.allclose(np.abs(np.abs(got) - np.abs(x)), nearest, rtol=0, atol=1e-15)
    assert np.all(np.sign(got) * np.sign(x) >= 0)


def test_encode_refuses_out_of_range():
    with pytest.raises(ValueError):
        quant.e4m3_encode(np.array([464.0]))


def test_quantize_blocks_maps_the_block_maximum_to_448_and_is_ragged_safe():
    rng = np.random.default_rng(9)
    x = rng.normal(0, 1, (300, 16)).astype(np.float32)
    x[128:256] = 0                                   # an all-zero block
    codes, scales = quant.quantize_blocks(x, 128)
    assert codes.shape == x.shape and scales.shape == (3,)
    assert scales[1] == 1.0 and np.all(codes[128:256] == 0)
    for b, rows in enumerate((slice(0, 128), slice(256, 300))):
        blk = b * 2
        assert scales[blk] == np.float32(np.abs(x[rows]).max() / np.float32(448.0))
        assert np.abs(quant.e4m3_decode(codes[rows])).max() == 448.0
    back = quant.dequantize_blocks(codes, scales, 128)
    # relative error of a normal E4M3 value is at most 2^-4; values below the block's 2^-6 * scale are subnormal
    err = np.abs(back - x)
    per_row_scale = np.repeat(scales.astype(np.float64), 128)[:300, None]
    assert np.all(err <= np.maximum(np.abs(x) * 2.0 ** -4, per_row_scale * 2.0 ** -10) * (1 + 1e-6))
