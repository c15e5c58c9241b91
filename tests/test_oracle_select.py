"""Pins of the selection oracle (oracle/select_oracle.py): the normal equations against
the pinned assembly oracle and brute force, the LASSO solver against closed forms and a
library solver, the regression scales against a library least squares, and Alg. 1 on
problems whose answer is known."""
import importlib.util
import os

import numpy as np
import pytest


def _selection_oracle():
    # the mutation test (test_oracle_mutations.py) points this at a deliberately broken copy
    path = os.environ.get("SR_SELECT_ORACLE_SRC")
    if not path:
        from oracle import select_oracle
        return select_oracle
    spec = importlib.util.spec_from_file_location("select_oracle_copy", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


so = _selection_oracle()


def _case(seed, n=1, c=2, H=9, W=11, L=6, k=3):
    rng = np.random.default_rng(seed)
    U = rng.normal(size=(n, c, H, W))
    coeff = rng.normal(size=(n, L, H, W))
    D = rng.normal(size=(L, k, k))
    return U, coeff, D


def test_responses_sum_to_the_assembled_image(oracle):
    # sum_l r_{p,l} is y_p of Eq. 2: ties the responses to the pinned assembly oracle
    U, coeff, D = _case(1, n=2, c=3, H=8, W=7, L=5, k=5)
    R = so.atom_responses(U, coeff, D)
    y = oracle.assemble(U, coeff, D)
    assert np.allclose(R.sum(axis=1).reshape(y.shape), y, rtol=0, atol=1e-12)
    # ... and with weights beta it is the selective assembly with gamma = beta
    beta = np.array([0.5, 0.0, -2.0, 1.0, 3.0])
    kept = np.nonzero(beta)[0].astype(np.int32)
    ys = oracle.assemble(U, coeff, D, kept=kept, gamma=beta[kept])
    assert np.allclose((R @ beta).reshape(ys.shape), ys, rtol=0, atol=1e-12)


def test_responses_brute_force_and_lattice():
    U, coeff, D = _case(2, n=1, c=1, H=6, W=5, L=3, k=3)
    R = so.atom_responses(U, coeff, D, stride=2).reshape(3, 3, 3)       # rows 0,2,4 x cols 0,2,4
    for iy, Y in enumerate((0, 2, 4)):
        for ix, X in enumerate((0, 2, 4)):
            for l in range(3):
                acc = 0.0
                for dy in range(3):
                    for dx in range(3):
                        yy, xx = min(max(Y + dy - 1, 0), 5), min(max(X + dx - 1, 0), 4)
                        acc += D[l, dy, dx] * U[0, 0, yy, xx]
                assert abs(R[iy, ix, l] - coeff[0, l, Y, X] * acc) < 1e-13


def test_normal_equations_give_the_residual_of_any_beta():
    U, coeff, D = _case(3)
    rng = np.random.default_rng(30)
    target = rng.normal(size=U.shape)
    G, b, hh, M = so.normal_equations(U, coeff, D, target, stride=1)
    assert M == U.size and G.shape == (6, 6) and np.allclose(G, G.T)
    R = so.atom_responses(U, coeff, D)
    for _ in range(3):
        beta = rng.normal(size=6)
        res = target.reshape(-1) - R @ beta
        assert np.isclose(hh - 2 * b @ beta + beta @ G @ beta, res @ res, rtol=1e-11)
    assert np.isclose(so.objective(G, b, hh, M, np.zeros(6), 0.3), hh / M)


def _regression(seed, M=400, L=8):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(M, L)) * rng.uniform(0.5, 2.0, size=L)
    w = rng.normal(size=L) * (rng.uniform(size=L) < 0.5)
    y = X @ w + 0.1 * rng.normal(size=M)
    return X, y, X.T @ X, X.T @ y, float(y @ y), M


def test_lasso_closed_forms():
    X, y, G, b, hh, M = _regression(4)
    assert np.allclose(so.lasso_cd(G, b, M, 0.0), np.linalg.lstsq(X, y, rcond=None)[0], atol=1e-9)
    lam_max = 2.0 * np.abs(b).max() / M                       # above it the zero vector is optimal
    assert not so.lasso_cd(G, b, M, lam_max * 1.0001).any()
    assert so.lasso_cd(G, b, M, lam_max * 0.99).any()
    # orthogonal design: plain soft thresholding of the least-squares solution
    Q, _ = np.linalg.qr(np.random.default_rng(5).normal(size=(50, 4)))
    yq = np.random.default_rng(6).normal(size=50)
    bq = Q.T @ yq
    lam = 0.02
    want = np.sign(bq) * np.maximum(np.abs(bq) - lam * 50 / 2, 0.0)
    assert np.allclose(so.lasso_cd(Q.T @ Q, bq, 50, lam), want, atol=1e-12)


def test_lasso_against_a_library_solver():
    sk = pytest.importorskip("sklearn.linear_model")
    for seed, lam in ((7, 0.05), (8, 0.3), (9, 1.0)):
        X, y, G, b, hh, M = _regression(seed)
        # the library minimises (1/2M)|y - Xw|^2 + a|w|_1: the same problem with a = lam/2
        ref = sk.Lasso(alpha=lam / 2, fit_intercept=False, tol=1e-14, max_iter=200000).fit(X, y).coef_
        mine = so.lasso_cd(G, b, M, lam)
        assert np.allclose(mine, ref, atol=1e-7)
        assert np.array_equal(mine != 0, ref != 0)
        # and it is a minimiser: no coordinate perturbation improves the objective
        f0 = so.objective(G, b, hh, M, mine, lam)
        for j in range(len(b)):
            for d in (-1e-4, 1e-4):
                p = mine.copy(); p[j] += d
                assert so.objective(G, b, hh, M, p, lam) >= f0 - 1e-15


def test_regression_scales_are_least_squares():
    X, y, G, b, hh, M = _regression(10)
    kept = [6, 1, 4]
    assert np.allclose(so.regression_scales(G, b, kept), np.linalg.lstsq(X[:, kept], y, rcond=None)[0], atol=1e-10)


def test_selection_recovers_a_planted_subset(oracle):
    # the target IS the selective assembly with 3 of 12 atoms and known scales:
    # Alg. 1 at alpha = 3/12 must return exactly those atoms and scales
    U, coeff, D = _case(11, n=2, c=2, H=12, W=10, L=12, k=3)
    planted = np.array([2, 7, 9], dtype=np.int32)
    scales = np.array([1.5, -0.75, 2.0])
    target = oracle.assemble(U, coeff, D, kept=planted, gamma=scales)
    G, b, hh, M = so.normal_equations(U, coeff, D, target)
    kept, gamma, lam = so.select_atoms(G, b, hh, M, alpha=3 / 12, delta_alpha=0.25)
    assert np.array_equal(kept, planted)
    assert np.allclose(gamma, scales, atol=1e-8)
    # one round straight to the target gives the same answer
    kept1, gamma1, _ = so.select_atoms(G, b, hh, M, alpha=3 / 12, delta_alpha=1.0)
    assert np.array_equal(kept1, planted) and np.allclose(gamma1, scales, atol=1e-8)
    # with the bisection switched off (eps = 1) the doubling alone must stop at the first
    # lambda that leaves at most alpha*L atoms: here the very first, which leaves these 3
    kept2, gamma2, lam2 = so.select_atoms(G, b, hh, M, alpha=3 / 12, delta_alpha=1.0, lam0=1e-6, eps=1.0)
    assert np.array_equal(kept2, planted) and np.allclose(gamma2, scales, atol=1e-8) and lam2 == 1e-6


def test_selection_keeps_at_most_alpha_L_and_never_raises_the_error_of_dropping_at_random():
    X, y, G, b, hh, M = _regression(12, M=600, L=20)
    for alpha in (0.5, 0.25, 0.1):
        kept, gamma, lam = so.select_atoms(G, b, hh, M, alpha=alpha, delta_alpha=0.25)
        assert 1 <= len(kept) <= alpha * 20 + 1e-9 and lam > 0
        assert np.array_equal(kept, np.sort(kept)) and len(set(kept.tolist())) == len(kept)
        full = np.zeros(20); full[kept] = gamma
        err = so.objective(G, b, hh, M, full, 0.0)
        # gamma is the least-squares fit on the kept atoms of the ORIGINAL responses
        assert np.allclose(gamma, np.linalg.lstsq(X[:, kept], y, rcond=None)[0], atol=1e-7)
        rng = np.random.default_rng(13)
        worse = 0
        for _ in range(20):
            rnd = np.sort(rng.choice(20, size=len(kept), replace=False))
            g = np.linalg.lstsq(X[:, rnd], y, rcond=None)[0]
            f = np.zeros(20); f[rnd] = g
            worse += so.objective(G, b, hh, M, f, 0.0) >= err - 1e-12
        assert worse >= 18                                     # the selected subset beats random ones
