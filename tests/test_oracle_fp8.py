"""Pins for the oracle's E4M3 encode/decode (OCP 8-bit floating point format), CPU only."""
import numpy as np

from oracle import vfm_oracle as orc


def test_decode_values_of_the_published_format():
    d = orc.fp8_e4m3_decode
    assert d(0x00) == 0.0 and d(0x38) == 1.0 and d(0x40) == 2.0 and d(0x44) == 3.0
    assert d(0x7E) == 448.0 and d(0xFE) == -448.0          # largest finite
    assert d(0x08) == 2.0 ** -6                             # smallest normal
    assert d(0x01) == 2.0 ** -9 and d(0x07) == 7 * 2.0 ** -9   # subnormals
    assert np.isnan(d(0x7F)) and np.isnan(d(0xFF))
    assert d(0x80) == 0.0 and np.signbit(d(0x80))
    # every binade holds 8 equally spaced values: 1, 1.125, ..., 1.875
    np.testing.assert_array_equal(d(np.arange(0x38, 0x40)), 1.0 + np.arange(8) / 8.0)


def test_decode_is_strictly_increasing_over_the_finite_codes():
    v = orc.fp8_e4m3_decode(np.arange(0x7F))
    assert np.all(np.diff(v) > 0)


def test_encode_inverts_decode_on_every_finite_code():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    back = orc.fp8_e4m3_encode(orc.fp8_e4m3_decode(codes))
    np.testing.assert_array_equal(back, codes)


def test_ties_go_to_the_even_code_and_large_values_saturate():
    e = orc.fp8_e4m3_encode
    assert e(17.0) == 0x58 and e(19.0) == 0x5A               # 16|18 -> 16 ; 18|20 -> 20
    assert e(1.0625) == 0x38 and e(1.1875) == 0x3A
    assert e(2.0 ** -10) == 0x00 and e(1.5 * 2.0 ** -10) == 0x01
    assert e(464.0) == 0x7E and e(1e9) == 0x7E and e(-np.inf) == 0xFE
    assert e(np.nan) == 0x7F
    assert e(0.3) == 0x2A and e(-0.3) == 0xAA


def test_encode_is_nearest():
    x = np.random.default_rng(0).standard_normal(20000) * 40.0
    q = orc.fp8_e4m3_decode(orc.fp8_e4m3_encode(x))
    grid = orc.fp8_e4m3_decode(np.arange(0x7F))
    grid = np.concatenate([-grid[::-1], grid])
    best = np.min(np.abs(np.clip(x, -448, 448)[:, None] - grid[None, :]), axis=1)
    np.testing.assert_allclose(np.abs(np.clip(x, -448, 448) - q), best, rtol=0, atol=0)


# ---------------------------------------------------------- per-tile power-of-two scales
def test_tile_exponent_is_the_largest_that_fits_by_brute_force():
    rng = np.random.default_rng(5)
    amax = np.concatenate([np.abs(rng.standard_normal(200)) * 10.0 ** rng.integers(-6, 7, 200),
                           [448.0, 448.0 * 2 ** -5, 448.0 * 2 ** 7, np.nextafter(448.0, 1e9), np.nextafter(448.0, 0.0),
                            224.0, 1.0, 1.75, np.nextafter(1.75, 2.0), 3.5e-5]])
    got = orc.fp8_tile_exponent(amax)
    for a, e in zip(amax, got):
        fits = [k for k in range(-130, 131) if a * 2.0 ** k <= 448.0]      # plain search
        assert int(e) == max(fits), (a, e)
        assert a * 2.0 ** int(e) > 224.0                                  # the top binade of E4M3 is used


def test_tile_exponent_special_cases():
    assert orc.fp8_tile_exponent(0.0) == 0
    assert orc.fp8_tile_exponent(448.0) == 0 and orc.fp8_tile_exponent(449.0) == -1
    assert orc.fp8_tile_exponent(1e-60) == 120 and orc.fp8_tile_exponent(1e60) == -120
    assert orc.fp8_tile_exponent(-3.0) == orc.fp8_tile_exponent(3.0) == 7    # 3 * 128 = 384 <= 448 < 768


def test_scaled_tile_round_trip_error_is_relative_to_the_tile():
    # storing x * 2**e and reading decode * 2**-e: error at most half an E4M3 step of the top binade,
    # 2**-4 of the tile's largest magnitude, however small or large the tile's values are
    rng = np.random.default_rng(6)
    for mag in (1e-4, 1.0, 3e4):
        x = rng.standard_normal(4096) * mag
        e = int(orc.fp8_tile_exponent(np.abs(x).max()))
        back = orc.fp8_e4m3_decode(orc.fp8_e4m3_encode(x * 2.0 ** e)) * 2.0 ** -e
        assert np.max(np.abs(back - x)) <= 2.0 ** -4 * np.abs(x).max()
