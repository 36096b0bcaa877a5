"""Pins for the stage-1 oracle (bilinear resize + normalise): closed forms, special
cases and brute force with exact rationals.  The paper (Section III-A) prints no
numeric example for this stage."""
from fractions import Fraction
from math import floor

import numpy as np
import pytest

from oracle import resize_bilinear_u8, normalize_lut, preprocess


def _rng_img(h, w, seed):
    return np.random.default_rng(seed).integers(0, 256, (h, w, 3), dtype=np.uint8)


def test_identity_resize_is_exact():
    img = _rng_img(17, 23, 0)
    assert np.array_equal(resize_bilinear_u8(img, 23, 17), img)


def test_constant_image_stays_constant():
    img = np.full((11, 13, 3), 201, dtype=np.uint8)
    for (wo, ho) in ((5, 4), (26, 22), (7, 31)):
        assert np.all(resize_bilinear_u8(img, wo, ho) == 201)


def test_exact_2to1_is_round_half_up_block_mean():
    img = _rng_img(12, 16, 1)
    out = resize_bilinear_u8(img, 8, 6)
    blk = img.astype(np.int64).reshape(6, 2, 8, 2, 3).sum(axis=(1, 3))
    assert np.array_equal(out, ((blk + 2) // 4).astype(np.uint8))


def test_horizontal_ramp_stays_monotone_and_rowwise_equal():
    ramp = np.tile(np.arange(0, 256, 4, dtype=np.uint8)[None, :, None], (9, 1, 3))
    out = resize_bilinear_u8(ramp, 29, 5).astype(int)
    assert np.all(np.diff(out[:, :, 0], axis=1) >= 0)
    assert np.all(out == out[0:1])
    assert out[0, 0, 0] >= 0 and out[0, -1, 0] <= 252


def _brute_pixel(img, X, Y, ch, wo, ho):
    """Textbook bilinear at half-pixel centres with exact rationals, edge clamp,
    round half up."""
    hi, wi, _ = img.shape
    sx = (Fraction(2 * X + 1, 2)) * Fraction(wi, wo) - Fraction(1, 2)
    sy = (Fraction(2 * Y + 1, 2)) * Fraction(hi, ho) - Fraction(1, 2)
    sx = min(max(sx, Fraction(0)), Fraction(wi - 1))
    sy = min(max(sy, Fraction(0)), Fraction(hi - 1))
    x0, y0 = floor(sx), floor(sy)
    fx, fy = sx - x0, sy - y0
    x1, y1 = min(x0 + 1, wi - 1), min(y0 + 1, hi - 1)
    v = ((1 - fx) * (1 - fy) * int(img[y0, x0, ch]) + fx * (1 - fy) * int(img[y0, x1, ch])
         + (1 - fx) * fy * int(img[y1, x0, ch]) + fx * fy * int(img[y1, x1, ch]))
    return floor(v + Fraction(1, 2))


@pytest.mark.parametrize("hi,wi,ho,wo", [(8, 8, 3, 5), (5, 7, 8, 8), (6, 9, 6, 4),
                                          (7, 3, 2, 9), (8, 6, 5, 5), (1, 4, 3, 7)])
def test_against_exact_rational_brute_force(hi, wi, ho, wo):
    img = _rng_img(hi, wi, hi * 100 + wi)
    out = resize_bilinear_u8(img, wo, ho)
    for Y in range(ho):
        for X in range(wo):
            for ch in range(3):
                assert out[Y, X, ch] == _brute_pixel(img, X, Y, ch, wo, ho), (X, Y, ch)


def test_transposed_input_gives_transposed_output():
    img = _rng_img(9, 14, 5)
    a = resize_bilinear_u8(img, 6, 4)
    b = resize_bilinear_u8(np.ascontiguousarray(img.transpose(1, 0, 2)), 4, 6)
    assert np.array_equal(a, b.transpose(1, 0, 2))


def test_lut_endpoints_and_monotone():
    lut = normalize_lut(0.5, 0.25, fp16=False)
    assert lut[0] == -2.0 and lut[255] == 2.0
    assert np.all(np.diff(lut) > 0)
    assert lut.dtype == np.float32
    # midpoint: (128/255 - 0.5)/0.25 = 2/255 * ... = 4*(128/255) - 2
    assert lut[128] == np.float32(4.0 * (128.0 / 255.0) - 2.0)
    lut16 = normalize_lut(0.5, 0.25, fp16=True)
    assert lut16[0] == -2.0 and lut16[255] == 2.0
    assert np.all(np.diff(lut16) >= 0)
    assert np.array_equal(lut16, lut16.astype(np.float16).astype(np.float32))
    assert np.max(np.abs(lut16 - lut)) <= 2.0 ** -10        # half ulp at magnitude <= 2


def test_preprocess_layout_is_planar_and_uses_lut():
    img = _rng_img(10, 12, 7)
    q, planar = preprocess(img, 12, 10, 0.5, 0.25, fp16=False)
    assert np.array_equal(q, img)
    assert planar.shape == (3, 10, 12)
    lut = normalize_lut(0.5, 0.25, False)
    assert planar[1, 3, 4] == lut[img[3, 4, 1]]
    assert planar[2, 9, 11] == lut[img[9, 11, 2]]
