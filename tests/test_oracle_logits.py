"""Pins of the oracle's logits form (an extension, not in the paper: the coefficients are the per-pixel softmax
over the atoms of stored logits, the exponentials rounded to binary16 before the sum):
  * a hand-worked pixel with exact values (tests/golden/logits_example.txt),
  * a closed form: logits that are logarithms of integers give the integers over their sum,
  * two libraries' softmax (scipy, torch) for the unrounded form, on every stored type,
  * the rounding: numpy's binary16 cast over doubles of every binade, ties and subnormals included, and, in
    the rounded form, every coefficient over the pixel's largest one IS the binary16 value of exp(z - max),
  * invariants: the coefficients of a pixel add up to one, a common shift of a pixel's logits changes nothing,
    logits far outside exp's range stay finite, each pixel is normalised by itself (and over the atoms),
  * the whole path: logits give what their coefficients, computed here another way, give."""
import os
from fractions import Fraction

import numpy as np
import pytest


def test_hand_worked_pixel(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "logits_example.txt")
    rows = [line.split() for line in open(path) if line.strip() and not line.startswith("#")]
    z = np.log(np.array([float(v) for v in rows[0]])).reshape(1, 4, 1, 1)
    num, den = [int(v) for v in rows[2]], int(rows[3][0])
    for rounded in (True, False):
        got = oracle.softmax_logits(z, round_half=rounded).reshape(-1)
        want = np.array([float(Fraction(v, den)) for v in num])
        assert np.max(np.abs(got - want)) < 1e-15
    # the exponentials of line 2 are the coefficients over the largest one
    got = oracle.softmax_logits(z).reshape(-1)
    assert np.allclose(got / got.max(), [float(v) for v in rows[1]], rtol=1e-15, atol=0)


def test_logarithms_of_integers_give_the_integers_over_their_sum(oracle):
    rng = np.random.default_rng(11)
    p = rng.integers(1, 50, size=(2, 7, 3, 4)).astype(np.float64)             # [N][L][H][W]
    got = oracle.softmax_logits(np.log(p), round_half=False)
    assert np.max(np.abs(got - p / p.sum(axis=1, keepdims=True))) < 1e-14


@pytest.mark.parametrize("dtype", [np.float64, np.float32, np.float16])
def test_unrounded_form_is_the_library_softmax(oracle, dtype):
    import scipy.special
    import torch
    rng = np.random.default_rng(12)
    z = (2.0 * rng.standard_normal((2, 9, 5, 6))).astype(dtype)
    got = oracle.softmax_logits(z, round_half=False)
    assert np.max(np.abs(got - scipy.special.softmax(z.astype(np.float64), axis=1))) < 1e-15
    assert np.max(np.abs(got - torch.softmax(torch.from_numpy(z.astype(np.float64)), dim=1).numpy())) < 1e-15


def test_stored_bfloat16_and_e4m3_logits_are_widened_first(oracle):
    rng = np.random.default_rng(13)
    for dtype, widen in ((np.uint16, oracle.bf16_to_double), (np.uint8, oracle.e4m3_to_double)):
        codes = rng.integers(0, 0x78 if dtype == np.uint8 else 0x4100, size=(1, 5, 3, 4)).astype(dtype)   # finite, modest values
        z = np.vectorize(widen)(codes)
        assert np.array_equal(oracle.softmax_logits(codes, round_half=False), oracle.softmax_logits(z, round_half=False))


def test_rounding_is_the_library_binary16_cast(oracle):
    rng = np.random.default_rng(14)
    v = np.concatenate([
        rng.random(4000) * np.exp2(rng.integers(-26, 1, size=4000)),              # every binade down to below the smallest subnormal
        (np.arange(2048, 4096) + 0.5) * 2.0 ** -12,                                # every tie of one binade: halves go to the even neighbour
        (np.arange(0, 64) + 0.5) * 2.0 ** -24,                                     # ties between subnormals
        [1.0, 0.5, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 0.0, 1.0 - 2.0 ** -12, 1.0 - 2.0 ** -13]])
    got = np.array([oracle.round_to_half(x) for x in v])
    assert np.array_equal(got, v.astype(np.float16).astype(np.float64))
    assert np.array_equal(np.array([oracle.round_to_half(-x) for x in v]), -got)


def test_rounded_form_divides_binary16_exponentials(oracle):
    rng = np.random.default_rng(15)
    z = (2.0 * rng.standard_normal((1, 72, 6, 7))).astype(np.float16)
    got = oracle.softmax_logits(z)
    z64 = z.astype(np.float64)
    e = np.exp(z64 - z64.max(axis=1, keepdims=True)).astype(np.float16).astype(np.float64)   # library exp, library cast
    want = e / e.sum(axis=1, keepdims=True)
    assert np.max(np.abs(got - want)) < 1e-15
    ratio = got / got.max(axis=1, keepdims=True)                     # the largest exponential is exactly 1
    assert np.max(np.abs(ratio - e)) < 1e-15
    plain = oracle.softmax_logits(z, round_half=False)
    err = np.abs(got - plain)
    assert err.max() > 1e-7                                          # rounded ...
    assert np.all(err <= 2.0 ** -10 * plain + 2.0 ** -25)            # ... by no more than binary16 rounds (2^-11 relative in a term and in the sum; 2^-25 below 2^-14)


def test_invariants(oracle):
    rng = np.random.default_rng(16)
    z = rng.integers(-40, 40, size=(2, 8, 4, 5)).astype(np.float32) / 8.0          # multiples of 1/8: shifts below are exact
    for rounded in (True, False):
        got = oracle.softmax_logits(z, round_half=rounded)
        assert np.max(np.abs(got.sum(axis=1) - 1.0)) < 1e-15
        shift = rng.integers(-16, 16, size=(2, 1, 4, 5)).astype(np.float32)       # one shift per pixel
        assert np.array_equal(oracle.softmax_logits(z + shift, round_half=rounded), got)
        # a pixel is normalised by itself: changing another pixel's logits leaves it alone
        z2 = z.copy()
        z2[0, :, 1, 2] += rng.standard_normal(8).astype(np.float32)
        got2 = oracle.softmax_logits(z2, round_half=rounded)
        mask = np.ones(got.shape, dtype=bool)
        mask[0, :, 1, 2] = False
        assert np.array_equal(got2[mask], got[mask]) and not np.array_equal(got2[0, :, 1, 2], got[0, :, 1, 2])
    big = np.array([800.0, 799.0, -800.0, 0.0]).reshape(1, 4, 1, 1)               # exp(800) is not a double
    got = oracle.softmax_logits(big, round_half=False).reshape(-1)
    assert np.all(np.isfinite(got)) and abs(got[0] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-15 and got[2] == 0.0 and got[3] == 0.0
    two = np.array([0.3, -1.1]).reshape(1, 2, 1, 1)                               # two atoms: the logistic function
    assert abs(oracle.softmax_logits(two, round_half=False)[0, 0, 0, 0] - 1.0 / (1.0 + np.exp(-1.4))) < 1e-15


def test_whole_path_with_logits(oracle):
    rng = np.random.default_rng(17)
    lr = rng.random((1, 2, 4, 5)).astype(np.float32)
    D = rng.standard_normal((6, 3, 3)).astype(np.float32)
    z = rng.standard_normal((1, 6, 8, 10)).astype(np.float16)
    z64 = z.astype(np.float64)
    e = np.exp(z64 - z64.max(axis=1, keepdims=True)).astype(np.float16).astype(np.float64)
    phi = e / e.sum(axis=1, keepdims=True)
    a = oracle.dict_assemble(lr, z, D, 2, logits=True)
    b = oracle.dict_assemble(lr, phi, D, 2)
    assert np.max(np.abs(a - b)) < 1e-14
    assert np.max(np.abs(a - oracle.dict_assemble(lr, z, D, 2))) > 1e-2           # logits are not coefficients
