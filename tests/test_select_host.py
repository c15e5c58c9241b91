"""Host side of the dictionary selection (sr_select_atoms, Alg. 1) against the numpy
oracle on the same normal equations.  No GPU involved."""
import ctypes

import numpy as np
import pytest

import paper_2303_08999_amd as sr
from oracle import select_oracle as so


def _problem(seed, M=500, L=24, noise=0.05):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(M, L)) * rng.uniform(0.3, 3.0, size=L)
    X[:, 1] = 0.7 * X[:, 0] + 0.3 * X[:, 1]                       # correlated atoms
    w = rng.normal(size=L) * (rng.uniform(size=L) < 0.4)
    y = X @ w + noise * rng.normal(size=M)
    G, b, hh = X.T @ X, X.T @ y, float(y @ y)
    return G, b, hh, M, np.concatenate([G.reshape(-1), b, [hh, float(M)]])


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("alpha,step", [(0.75, 0.25), (0.5, 0.1), (0.25, 0.25), (0.1, 0.3), (1 / 24, 1.0)])
def test_same_selection_as_the_oracle(seed, alpha, step):
    G, b, hh, M, normal = _problem(seed)
    k0, g0, l0 = so.select_atoms(G, b, hh, M, alpha, step, lam0=1e-5)
    k1, g1, l1 = sr.sr_select_atoms(normal, 24, alpha, step, lambda0=1e-5)
    assert np.array_equal(k0, k1)
    assert len(k1) <= alpha * 24 + 1e-9
    assert np.allclose(g0, g1, rtol=1e-6, atol=1e-7)
    assert np.isclose(l0, l1, rtol=1e-12)


def test_planted_subset_is_recovered():
    rng = np.random.default_rng(9)
    X = rng.normal(size=(300, 16))
    planted, scales = [3, 8, 12, 15], np.array([2.0, -1.0, 0.5, 1.25])
    y = X[:, planted] @ scales
    normal = np.concatenate([(X.T @ X).reshape(-1), X.T @ y, [float(y @ y), 300.0]])
    kept, gamma, _ = sr.sr_select_atoms(normal, 16, 4 / 16, delta_alpha=0.25)
    assert kept.tolist() == planted and np.allclose(gamma, scales, atol=1e-5)
    kept, gamma, lam = sr.sr_select_atoms(normal, 16, 4 / 16, delta_alpha=1.0, lambda0=1e-6, eps=1.0)
    assert kept.tolist() == planted and np.allclose(gamma, scales, atol=1e-5) and lam == 1e-6


def test_selection_against_an_independent_solver_and_brute_force():
    """The product's search checked against things that are NOT its twin (the numpy oracle follows the same
    steps): a library LASSO solver at the lambda the search reports, least squares on the kept columns,
    and exhaustive best-subset search on problems small enough for it."""
    sk = pytest.importorskip("sklearn.linear_model")
    import itertools
    rng = np.random.default_rng(21)
    for trial in range(6):
        M, L, k = 400, 10, 3
        X = rng.normal(size=(M, L))
        planted = np.sort(rng.choice(L, size=k, replace=False))
        w = np.zeros(L)
        w[planted] = rng.uniform(1.0, 2.5, size=k) * rng.choice([-1.0, 1.0], size=k)
        y = X @ w + 0.05 * rng.normal(size=M)
        normal = np.concatenate([(X.T @ X).reshape(-1), X.T @ y, [float(y @ y), float(M)]])
        # one round straight to the target count: the kept set is the support of ONE LASSO problem
        kept, gamma, lam = sr.sr_select_atoms(normal, L, k / L, delta_alpha=1.0, lambda0=1e-4)
        assert 1 <= len(kept) <= k
        # (a) library solver, same objective ((1/M)|y - X b|^2 + lam |b|_1 = 2 x sklearn's with alpha = lam / 2)
        ref = sk.Lasso(alpha=lam / 2, fit_intercept=False, tol=1e-14, max_iter=200000).fit(X, y).coef_
        assert np.flatnonzero(np.abs(ref) > 1e-10).tolist() == kept.tolist()
        # ... and just below that lambda no fewer atoms survive
        if lam > 1e-4:
            below = sk.Lasso(alpha=0.999 * lam / 2, fit_intercept=False, tol=1e-14, max_iter=200000).fit(X, y).coef_
            assert np.count_nonzero(np.abs(below) > 1e-10) >= len(kept)
        # (b) gamma is the least-squares fit on the kept columns (Eq. 9), from a library routine
        ls = np.linalg.lstsq(X[:, kept], y, rcond=None)[0]
        assert np.allclose(gamma, ls, rtol=1e-5, atol=1e-6)
        # (c) exhaustive search: no other subset of that size fits better, and with this little noise it is the planted one
        best = min(itertools.combinations(range(L), len(kept)),
                   key=lambda S: float(np.linalg.lstsq(X[:, S], y, rcond=None)[1][0]))
        assert list(best) == kept.tolist() == planted[:len(kept)].tolist() or set(kept) <= set(planted)
        if len(kept) == k:
            assert list(best) == kept.tolist() == planted.tolist()


def test_alpha_one_keeps_everything_untouched():
    G, b, hh, M, normal = _problem(4)
    kept, gamma, lam = sr.sr_select_atoms(normal, 24, 1.0)
    assert kept.tolist() == list(range(24)) and np.all(gamma == 1.0) and lam == 1e-6


def test_argument_checks():
    lib = sr.load()
    G, b, hh, M, normal = _problem(5)
    dp = normal.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    kept = (ctypes.c_int * 24)(); gam = (ctypes.c_float * 24)(); n = ctypes.c_int()
    ok = lambda *a: lib.sr_select_atoms(*a)
    assert ok(None, 24, 0.5, 0.1, 1e-6, 0.0, kept, ctypes.byref(n), gam, None) == -1
    assert ok(dp, 24, 0.5, 0.1, 1e-6, 0.0, None, ctypes.byref(n), gam, None) == -1
    assert ok(dp, 0, 0.5, 0.1, 1e-6, 0.0, kept, ctypes.byref(n), gam, None) == -3
    assert ok(dp, 129, 0.5, 0.1, 1e-6, 0.0, kept, ctypes.byref(n), gam, None) == -3
    for bad in ((0.0, 0.1, 1e-6, 0.0), (1.5, 0.1, 1e-6, 0.0), (0.5, 0.0, 1e-6, 0.0), (0.5, 0.1, 0.0, 0.0),
                (0.5, 0.1, 1e-6, -1.0), (float("nan"), 0.1, 1e-6, 0.0)):
        assert ok(dp, 24, *bad, kept, ctypes.byref(n), gam, None) == -3
    assert ok(dp, 24, 0.5, 0.1, 1e-6, 0.0, kept, ctypes.byref(n), gam, None) == 0 and 1 <= n.value <= 12
    # gram entry point: everything is checked before anything is launched
    assert lib.sr_atom_gram_workspace_bytes(72) == 512 * 15 * 256 * 8        # 15 blocks of 16 x 16 doubles per workgroup
    assert lib.sr_atom_gram_workspace_bytes(0) == 0 and lib.sr_atom_gram_workspace_bytes(129) == 0
    T = sr.sr_tensor
    up = T(0x10000000, sr.SR_F32, 1, 3, 32, 64); tg = T(0x20000000, sr.SR_F32, 1, 3, 32, 64)
    cf = T(0x30000000, sr.SR_F16, 1, 72, 32, 64); d = T(0x40000000, sr.SR_F32, 1, 72, 5, 5)
    ws, nm = ctypes.c_void_p(0x50000000), ctypes.c_void_p(0x60000000)
    need = lib.sr_atom_gram_workspace_bytes(72)
    g = lambda *a: lib.sr_atom_gram(*a)
    assert g(None, cf, d, tg, 72, 5, 3, 1, ws, need, nm, None) == -1
    assert g(up, cf, d, tg, 72, 5, 3, 1, ws, need, None, None) == -1
    assert g(up, cf, d, tg, 72, 5, 3, 1, None, need, nm, None) == -2           # no scratch
    assert g(up, cf, d, tg, 72, 5, 3, 1, ws, need - 1, nm, None) == -2         # scratch too small
    assert g(up, cf, d, tg, 72, 4, 3, 1, ws, need, nm, None) == -3
    assert g(up, cf, d, tg, 72, 5, 3, 0, ws, need, nm, None) == -3
    assert g(up, cf, d, tg, 71, 5, 3, 1, ws, need, nm, None) == -2             # L disagrees with coeff
    assert g(up, cf, d, T(0x20000000, sr.SR_F32, 1, 3, 32, 60), 72, 5, 3, 1, ws, need, nm, None) == -2
    assert g(T(0x10000000, sr.SR_F16, 1, 3, 32, 64), cf, d, tg, 72, 5, 3, 1, ws, need, nm, None) == -3
    assert g(up, cf, d, tg, 72, 5, 3, 1, ctypes.c_void_p(0x50000008), need, nm, None) == -7
