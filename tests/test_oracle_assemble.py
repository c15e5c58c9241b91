"""Pins for the oracle's stages 3 + 4 (paper Eq. 2 / Eq. 3) and for the
compressed-dictionary form (section III-A).

The paper prints no worked numeric example of Eq. 2, so the pins are: delta
atoms (centred and off-centre), linearity, constant preservation, an
exact-rational evaluator in the other association, and a library
pad + unfold + einsum.
"""
import numpy as np
import pytest
import torch

from rational_brute import assemble_exact, to_fractions, upsample_exact


def _rand_case(seed, n=1, c=2, H=7, W=9, L=5, k=3):
    rng = np.random.default_rng(seed)
    U = rng.normal(size=(n, c, H, W))
    coeff = rng.normal(size=(n, L, H, W))
    D = rng.normal(size=(L, k, k))
    return U, coeff, D


@pytest.mark.parametrize("k", [3, 5, 7])
def test_centred_delta_atom_reproduces_the_upsampled_image(oracle, k):
    rng = np.random.default_rng(k)
    lr = rng.uniform(0, 1, size=(1, 3, 6, 5)).astype(np.float32)
    L = 4
    D = rng.normal(size=(L, k, k))
    D[2] = 0.0
    D[2, k // 2, k // 2] = 1.0
    coeff = np.zeros((1, L, 12, 10))
    coeff[:, 2] = 1.0
    out = oracle.dict_assemble(lr, coeff, D, 2)
    assert np.array_equal(out, oracle.bicubic(lr, 2))


@pytest.mark.parametrize("k,dy,dx", [(3, 0, 2), (5, 4, 1), (5, 0, 0), (7, 6, 3), (5, 2, 4)])
def test_off_centre_delta_pins_orientation_and_border(oracle, k, dy, dx):
    """A delta at tap (dy, dx) must read U[Y+dy-r][X+dx-r] with the index
    clamped to the HR image: correlation, row-major taps, replicate padding."""
    rng = np.random.default_rng(100 + k + dy)
    H, W = 9, 11
    U = rng.normal(size=(1, 2, H, W))
    D = np.zeros((1, k, k))
    D[0, dy, dx] = 1.0
    coeff = np.ones((1, 1, H, W))
    out = oracle.assemble(U, coeff, D)
    r = (k - 1) // 2
    yy = np.clip(np.arange(H) + dy - r, 0, H - 1)
    xx = np.clip(np.arange(W) + dx - r, 0, W - 1)
    assert np.array_equal(out, U[:, :, yy][:, :, :, xx])


def test_linear_in_coefficients_dictionary_and_image(oracle):
    U, c1, D = _rand_case(1)
    _, c2, D2 = _rand_case(2)
    U2 = np.random.default_rng(3).normal(size=U.shape)
    a, b = -1.75, 0.6
    f = oracle.assemble
    assert np.max(np.abs(f(U, a * c1 + b * c2, D) - (a * f(U, c1, D) + b * f(U, c2, D)))) < 1e-12
    assert np.max(np.abs(f(U, c1, a * D + b * D2) - (a * f(U, c1, D) + b * f(U, c1, D2)))) < 1e-12
    assert np.max(np.abs(f(a * U + b * U2, c1, D) - (a * f(U, c1, D) + b * f(U2, c1, D)))) < 1e-12


@pytest.mark.parametrize("scale", [2, 3, 4])
def test_constant_image_preserved_with_normalised_atoms_and_unit_sum(oracle, scale):
    rng = np.random.default_rng(7)
    L, k = 6, 5
    D = rng.normal(size=(L, k, k))
    D /= D.sum(axis=(1, 2), keepdims=True)
    logits = rng.normal(size=(1, L, 4 * scale, 5 * scale))
    coeff = np.exp(logits) / np.exp(logits).sum(axis=1, keepdims=True)
    lr = np.full((1, 3, 4, 5), 0.625)
    out = oracle.dict_assemble(lr, coeff, D, scale)
    assert np.max(np.abs(out - 0.625)) < 1e-13   # every pixel, borders included


def test_library_unfold_einsum(oracle):
    """Stages 3 + 4 as library calls: replicate-pad, unfold, contract."""
    n, c, H, W, L, k = 2, 3, 10, 13, 7, 5
    U, coeff, D = _rand_case(17, n, c, H, W, L, k)
    r = k // 2
    Ut = torch.from_numpy(U).reshape(n * c, 1, H, W)
    pad = torch.nn.functional.pad(Ut, (r, r, r, r), mode="replicate")
    B = torch.nn.functional.unfold(pad, k).reshape(n, c, k * k, H, W)
    F = torch.einsum("nlhw,lj->njhw", torch.from_numpy(coeff), torch.from_numpy(D).reshape(L, k * k))
    want = torch.einsum("njhw,ncjhw->nchw", F, B).numpy()
    assert np.max(np.abs(oracle.assemble(U, coeff, D) - want)) < 1e-12


@pytest.mark.parametrize("scale,k", [(2, 3), (3, 3), (4, 5)])
def test_exact_rational_whole_path_other_association(oracle, scale, k):
    rng = np.random.default_rng(40 + scale)
    h, w, L = 2, 3, 3
    lr = rng.integers(0, 64, size=(h, w)).astype(np.float64) / 64
    D = rng.integers(-8, 9, size=(L, k, k)).astype(np.float64) / 8
    coeff = rng.integers(-16, 17, size=(L, h * scale, w * scale)).astype(np.float64) / 16
    U = upsample_exact(to_fractions(lr), scale)
    exact = assemble_exact(U, to_fractions(coeff), to_fractions(D))
    want = np.array([[float(v) for v in row] for row in exact])
    got = oracle.dict_assemble(lr[None, None], coeff[None], D, scale)[0, 0]
    assert np.max(np.abs(got - want)) < 1e-13


def test_selective_forms(oracle):
    U, coeff, D = _rand_case(23, L=8)
    L = D.shape[0]
    dense = oracle.assemble(U, coeff, D)
    assert np.array_equal(oracle.assemble(U, coeff, D, kept=np.arange(L)), dense)
    kept = np.array([6, 1, 3])
    masked = np.zeros_like(coeff)
    masked[:, kept] = coeff[:, kept]
    sel = oracle.assemble(U, coeff, D, kept=kept)
    assert np.max(np.abs(sel - oracle.assemble(U, masked, D))) < 1e-12
    gamma = np.array([0.5, -2.0, 1.25])
    scaled = np.zeros_like(coeff)
    scaled[:, kept] = coeff[:, kept] * gamma[None, :, None, None]
    assert np.max(np.abs(oracle.assemble(U, coeff, D, kept=kept, gamma=gamma)
                         - oracle.assemble(U, scaled, D))) < 1e-12
    # exact rational check of the selective form too
    Uf = to_fractions(U[0, 0])
    exact = assemble_exact(Uf, to_fractions(coeff[0]), to_fractions(D), kept=list(kept),
                           gamma=[__import__("fractions").Fraction(float(g)) for g in gamma])
    want = np.array([[float(v) for v in row] for row in exact])
    assert np.max(np.abs(oracle.assemble(U, coeff, D, kept=kept, gamma=gamma)[0, 0] - want)) < 1e-12


def test_rows_and_points_agree_with_full(oracle):
    U, coeff, D = _rand_case(31, n=2, c=3, H=8, W=6, L=4, k=5)
    full = oracle.assemble(U, coeff, D)
    part = oracle.assemble(U, coeff, D, rows=(2, 5))
    assert np.array_equal(part[:, :, 2:5], full[:, :, 2:5])
    assert not part[:, :, :2].any() and not part[:, :, 5:].any()
    pts = [(0, 0, 0), (1, 7, 5), (0, 3, 2), (1, 0, 5)]
    got = oracle.assemble_points(U, coeff, D, pts)
    for row, (b, y, x) in zip(got, pts):
        assert np.array_equal(row, full[b, :, y, x])


def test_stored_fp16_and_fp32_coefficients_are_widened(oracle):
    U, coeff, D = _rand_case(37)
    c16 = coeff.astype(np.float16)
    assert np.array_equal(oracle.assemble(U, c16, D), oracle.assemble(U, c16.astype(np.float64), D))
    c32 = coeff.astype(np.float32)
    assert np.array_equal(oracle.assemble(U, c32, D), oracle.assemble(U, c32.astype(np.float64), D))


def test_bad_arguments_are_rejected(oracle):
    U, coeff, D = _rand_case(41)
    with pytest.raises(ValueError):
        oracle.assemble(U, coeff, D, kept=[0, 99])
    with pytest.raises(ValueError):
        oracle.assemble(U, coeff[:, :2], D)
    with pytest.raises(ValueError):
        oracle.assemble(U, coeff, np.zeros((5, 4, 4)))


def test_results_do_not_depend_on_the_thread_count(oracle):
    U, coeff, D = _rand_case(77, n=2, c=2, H=19, W=11, L=7, k=5)
    before = oracle.threads()
    try:
        assert oracle.set_threads(1) == 1
        one = oracle.assemble(U, coeff, D)
        assert oracle.set_threads(3) == 3
        three = oracle.assemble(U, coeff, D)
    finally:
        oracle.set_threads(before)
    assert np.array_equal(one, three)
