"""CPU oracle for the offline dictionary selection -- TEST INFRASTRUCTURE ONLY.

Plain numpy, double precision, the steps of the paper's dictionary selection
strategy (section III-A: Eq. 7 the relaxed LASSO objective, Alg. 1 the search
for the regularisation weight, Eq. 9 the regression scales gamma) in the
paper's order.  Only tests may import this module.

What the selection works on.  With the dictionary query and the filtering taken
together (Eq. 6), the image produced with selector beta is, for a sample p (one
HR pixel of one channel),

    y_p(beta) = sum_l beta_l * r_{p,l},      r_{p,l} = Phi_{p,l} * (D_l . B_p)

(r_{p,l} is "apply atom l to the neighbourhood, weight by the coefficient"), so
Eq. 7 is a LASSO regression of the ground-truth pixels on the per-atom
responses R = [r_{p,l}].  It only needs the normal equations
G = R^T R, b = R^T h, hh = h^T h and the sample count M.

Readings taken where the paper is silent or inconsistent:
  * the data term is averaged over the M samples (the paper writes 1/N with N
    the batch size; only the scale of lambda depends on it);
  * the samples are the pixels of a regular lattice (every `stride`-th row and
    column, all channels), a deterministic stand-in for the paper's random
    sampling;
  * the LASSO problems are solved by cyclic coordinate descent (the paper names
    no solver);
  * the bisection of Alg. 1 as printed moves the wrong bound (a sparser
    solution would raise lambda further); it is taken as ordinary bisection
    between the last lambda that left too many atoms and the first that did not;
  * the fine-tuning of the coefficient network between selection rounds is the
    regression of Eq. 9, as the paper proposes: the kept atoms' coefficients are
    rescaled by gamma, which here rescales the normal equations;
  * alpha_t is not stepped below the target alpha.
"""
from __future__ import annotations

import numpy as np


def atom_responses(U, coeff, dictionary, stride=1):
    """R[M][L] and the sample order: samples run over (image, channel, Y, X) with
    Y and X multiples of `stride`.  U [n][c][H][W] is the up-sampled image, coeff
    [n][L][H][W], dictionary [L][k][k]; patch taps outside the image read the
    nearest pixel (as everywhere in this build)."""
    U = np.asarray(U, dtype=np.float64)
    coeff = np.asarray(coeff)
    if coeff.dtype == np.uint8:                      # stored 8-bit E4M3 floats, widened by the assembly oracle's decoder
        from . import e4m3_to_double
        coeff = np.array([e4m3_to_double(b) for b in range(256)])[coeff]
    elif coeff.dtype == np.uint16:                   # stored bfloat16, likewise
        from . import bf16_to_double
        coeff = np.array([bf16_to_double(b) for b in range(65536)])[coeff]
    coeff = coeff.astype(np.float64)
    D = np.asarray(dictionary, dtype=np.float64)
    n, c, H, W = U.shape
    L, k, _ = D.shape
    r = (k - 1) // 2
    ys, xs = np.arange(0, H, stride), np.arange(0, W, stride)
    Up = np.pad(U, ((0, 0), (0, 0), (r, r), (r, r)), mode="edge")
    R = np.zeros((n, c, len(ys), len(xs), L))
    for dy in range(k):
        for dx in range(k):
            tap = Up[:, :, dy:dy + H, dx:dx + W][:, :, ys][:, :, :, xs]      # B_p[dy*k + dx]
            R += tap[..., None] * D[:, dy, dx]
    phi = coeff[:, :, ys][:, :, :, xs]                                       # [n][L][ny][nx]
    R *= np.moveaxis(phi, 1, -1)[:, None]
    return R.reshape(-1, L)


def normal_equations(U, coeff, dictionary, target, stride=1):
    """G = R^T R [L][L], b = R^T h [L], hh = h^T h, M = number of samples."""
    R = atom_responses(U, coeff, dictionary, stride)
    t = np.asarray(target, dtype=np.float64)
    H, W = t.shape[2], t.shape[3]
    h = t[:, :, np.arange(0, H, stride)][:, :, :, np.arange(0, W, stride)].reshape(-1)
    return R.T @ R, R.T @ h, float(h @ h), R.shape[0]


def objective(G, b, hh, M, beta, lam):
    """(1/M) |h - R beta|^2 + lam |beta|_1 from the normal equations (Eq. 7)."""
    beta = np.asarray(beta, dtype=np.float64)
    return (hh - 2.0 * b @ beta + beta @ G @ beta) / M + lam * np.abs(beta).sum()


def lasso_cd(G, b, M, lam, beta0=None, tol=1e-13, max_sweeps=100000):
    """argmin_beta (1/M)|h - R beta|^2 + lam |beta|_1 by cyclic coordinate descent:
    beta_j <- soft(b_j - sum_{k != j} G_jk beta_k, lam M / 2) / G_jj."""
    G = np.asarray(G, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    L = len(b)
    beta = np.ones(L) if beta0 is None else np.array(beta0, dtype=np.float64)
    thr = 0.5 * lam * M
    for _ in range(max_sweeps):
        dmax = 0.0
        for j in range(L):
            if G[j, j] <= 0.0:
                new = 0.0
            else:
                rho = b[j] - (G[j] @ beta - G[j, j] * beta[j])
                new = (rho - thr if rho > thr else (rho + thr if rho < -thr else 0.0)) / G[j, j]
            dmax = max(dmax, abs(new - beta[j]))
            beta[j] = new
        if dmax <= tol * max(1.0, np.abs(beta).max()):
            break
    return beta


def regression_scales(G, b, kept):
    """Eq. 9 on the kept atoms: gamma = argmin |h - sum_{l in kept} gamma_l r_l|^2,
    i.e. G_SS gamma = b_S (least squares if G_SS is singular)."""
    S = np.asarray(kept, dtype=np.int64)
    Gs, bs = np.asarray(G, dtype=np.float64)[np.ix_(S, S)], np.asarray(b, dtype=np.float64)[S]
    try:
        return np.linalg.solve(Gs, bs)
    except np.linalg.LinAlgError:
        return np.linalg.lstsq(Gs, bs, rcond=None)[0]


def select_atoms(G, b, hh, M, alpha, delta_alpha=0.1, lam0=1e-6, eps=0.0, max_bisect=60):
    """Alg. 1.  Returns (kept atom indices, ascending; their cumulative gamma;
    the lambda reached).  At most alpha*L atoms are kept."""
    G = np.array(G, dtype=np.float64)
    b = np.array(b, dtype=np.float64)
    L = len(b)
    active = np.arange(L)
    gamma_tot = np.ones(L)
    alpha_t, lam = 1.0, float(lam0)
    while alpha_t > alpha + 1e-12 and len(active) > 0:
        alpha_t = max(alpha, alpha_t - delta_alpha)
        want = alpha_t * L
        Ga, ba = G[np.ix_(active, active)], b[active]

        def solve(lm):
            bt = lasso_cd(Ga, ba, M, lm)
            return bt, int(np.count_nonzero(bt))

        # lambda doubles until few enough atoms survive
        lam_lo, lam_hi = 0.5 * lam, lam
        beta, cnt = solve(lam_hi)
        while cnt > want:
            lam_lo, lam_hi = lam_hi, 2.0 * lam_hi
            beta, cnt = solve(lam_hi)
        # bisection towards the target count, keeping a solution that meets it
        it = 0
        while abs(want - cnt) > eps * L and want - cnt >= 1.0 and it < max_bisect:
            mid = 0.5 * (lam_lo + lam_hi)
            bm, cm = solve(mid)
            if cm > want:
                lam_lo = mid
            else:
                lam_hi, beta, cnt = mid, bm, cm
            it += 1
        lam = lam_hi
        keep = np.nonzero(beta)[0]
        if len(keep) == 0:
            active = active[:0]
            break
        gam = regression_scales(Ga, ba, keep)
        S = active[keep]
        gamma_tot[S] *= gam
        # the kept atoms' coefficients are rescaled by gamma from here on
        G[np.ix_(S, S)] *= np.outer(gam, gam)
        b[S] *= gam
        active = S
    mask = np.zeros(L, dtype=bool)
    mask[active] = True
    gamma_tot[~mask] = 0.0
    return active.astype(np.int32), gamma_tot[active], lam
