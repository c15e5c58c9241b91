"""Pins for the oracle's stage 1 (upsampling; paper section II-B stage 1).

None of these re-types the oracle's formula: they use the hand-derived rational
phase table (tests/golden), polynomial reproduction (a property only a = -1/2
has), a library interpolator at that library's own constant, and invariants.
"""
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

from rational_brute import load_phase_table, upsample_exact, to_fractions


def test_half_decode_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


@pytest.mark.parametrize("scale", [2, 3, 4])
def test_phase_weights_match_golden_rationals(oracle, scale):
    table = load_phase_table()
    for Y in range(0, 5 * scale):
        p = Y % scale
        off, wts = table[(scale, p)]
        first, w = oracle.taps(Y, scale)
        assert first == (Y - p) // scale + off - 1
        for got, want in zip(w, wts):
            assert abs(got - float(want)) < 1e-14
        assert abs(sum(w) - 1.0) < 1e-14


def test_kernel_interpolates_and_has_compact_support(oracle):
    assert oracle.keys(0.0) == 1.0
    for t in (1.0, -1.0, 2.0, -2.0, 2.5, 7.0):
        assert abs(oracle.keys(t)) < 1e-15
    assert oracle.keys(0.3) == oracle.keys(-0.3)


@pytest.mark.parametrize("scale", [2, 3, 4])
def test_quadratic_reproduction_fixes_a_and_coordinates(oracle, scale):
    """Cubic convolution with a = -1/2 reproduces polynomials up to degree 2
    exactly (Keys 1981); no other a even reproduces a ramp.  Evaluated at the
    half-pixel source coordinates, away from the replicated border."""
    h, w = 12, 14
    yy, xx = np.mgrid[0:h, 0:w].astype(np.float64)

    def poly(y, x):
        return 0.3 + 0.7 * y - 0.45 * x + 0.05 * y * y + 0.11 * x * y - 0.08 * x * x

    lr = poly(yy, xx)[None, None]
    U = oracle.bicubic(lr, scale)[0, 0]
    Y, X = np.mgrid[0:h * scale, 0:w * scale].astype(np.float64)
    sy, sx = (Y + 0.5) / scale - 0.5, (X + 0.5) / scale - 0.5
    inner = (sy >= 1) & (sy <= h - 3) & (sx >= 1) & (sx <= w - 3)
    assert inner.sum() > 100
    assert np.max(np.abs(U - poly(sy, sx))[inner]) < 1e-11
    # and a different a must NOT reproduce even the linear part
    U75 = oracle.bicubic(lr, scale, a=-0.75)[0, 0]
    assert np.max(np.abs(U75 - poly(sy, sx))[inner]) > 1e-3


@pytest.mark.parametrize("scale", [2, 3, 4])
@pytest.mark.parametrize("shape", [(5, 7), (1, 9), (8, 1), (2, 2)])
def test_library_bicubic_at_its_own_constant(oracle, scale, shape):
    """torch's bicubic (align_corners=False) is the same interpolator with
    a = -0.75, half-pixel centres and clamped indices: it pins the tap order,
    the coordinate convention and the border rule, including tiny images."""
    rng = np.random.default_rng(11 + scale)
    lr = rng.uniform(-1, 2, size=(2, 3) + shape)
    want = torch.nn.functional.interpolate(torch.from_numpy(lr), scale_factor=scale,
                                           mode="bicubic", align_corners=False).numpy()
    got = oracle.bicubic(lr, scale, a=-0.75)
    assert got.shape == want.shape
    assert np.max(np.abs(got - want)) < 1e-12


def test_scale3_passes_lr_pixels_through(oracle):
    rng = np.random.default_rng(5)
    lr = rng.uniform(0, 1, size=(1, 2, 6, 5))
    U = oracle.bicubic(lr, 3)
    assert np.array_equal(U[:, :, 1::3, 1::3], lr)


@pytest.mark.parametrize("scale", [2, 3, 4])
def test_constant_image_stays_constant(oracle, scale):
    lr = np.full((1, 1, 4, 6), 0.3125)
    U = oracle.bicubic(lr, scale)
    assert np.max(np.abs(U - 0.3125)) < 1e-15


@pytest.mark.parametrize("scale", [2, 3, 4])
def test_exact_rational_upsample(oracle, scale):
    """Whole tiny image, borders included, against exact rational arithmetic
    built from the golden table (x2 and x4 weights are dyadic, so the oracle
    must be exact to the last bit there)."""
    rng = np.random.default_rng(3)
    lr = rng.integers(0, 256, size=(4, 5)).astype(np.float64) / 256.0
    exact = upsample_exact(to_fractions(lr), scale)
    got = oracle.bicubic(lr[None, None], scale)[0, 0]
    want = np.array([[float(v) for v in row] for row in exact])
    tol = 0.0 if scale in (2, 4) else 1e-15
    assert np.max(np.abs(got - want)) <= tol


def test_dtypes_are_widened_not_regenerated(oracle):
    rng = np.random.default_rng(9)
    lr16 = rng.uniform(0, 1, size=(1, 1, 5, 5)).astype(np.float16)
    a = oracle.bicubic(lr16, 2)
    b = oracle.bicubic(lr16.astype(np.float64), 2)
    c = oracle.bicubic(lr16.astype(np.float32), 2)
    assert np.array_equal(a, b) and np.array_equal(a, c)


def test_linear_in_the_image(oracle):
    rng = np.random.default_rng(21)
    x1, x2 = rng.normal(size=(2, 1, 1, 6, 6))
    lhs = oracle.bicubic(2.5 * x1 - 0.75 * x2, 4)
    rhs = 2.5 * oracle.bicubic(x1, 4) - 0.75 * oracle.bicubic(x2, 4)
    assert np.max(np.abs(lhs - rhs)) < 1e-13
