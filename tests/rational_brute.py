"""Exact-rational evaluator of the whole path for tiny inputs (test helper).

Deliberately the OTHER association from the oracle's: apply each of the L
dictionary filters to the upsampled neighbourhood, weight the L responses by the
pixel's coefficients, sum (the LAPAR-style statement of the path), where the
oracle folds the filter first (paper Eq. 2, ``F_i = Phi_i D`` then
``y_i = F_i B_i^T``).  Python ``fractions`` throughout, so the result is the
exact value both orders must reach.

The interpolator here is built from the golden phase table
(tests/golden/bicubic_phase_weights.txt), not from a kernel formula, so it does
not restate the oracle's arithmetic.
"""
from __future__ import annotations

import os
from fractions import Fraction as Fr

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                      "bicubic_phase_weights.txt")


def load_phase_table():
    table = {}
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if not line:
                continue
            s, p, off = int(line[0]), int(line[1]), int(line[2])
            table[(s, p)] = (off, [Fr(x) for x in line[3:7]])
    return table


def _clamp(v, lo, hi):
    return lo if v < lo else (hi if v > hi else v)


def upsample_exact(img, s, table=None):
    """img: h x w nested lists of Fractions -> (s*h) x (s*w) nested lists."""
    table = table or load_phase_table()
    h, w = len(img), len(img[0])

    def taps(Y):
        p = Y % s
        off, wts = table[(s, p)]
        return (Y - p) // s + off - 1, wts

    out = [[Fr(0)] * (s * w) for _ in range(s * h)]
    for Y in range(s * h):
        fy, wy = taps(Y)
        for X in range(s * w):
            fx, wx = taps(X)
            acc = Fr(0)
            for i in range(4):
                for j in range(4):
                    acc += wy[i] * wx[j] * img[_clamp(fy + i, 0, h - 1)][_clamp(fx + j, 0, w - 1)]
            out[Y][X] = acc
    return out


def assemble_exact(U, coeff, atoms, kept=None, gamma=None):
    """U: H x W Fractions (one channel); coeff: L x H x W; atoms: L x k x k.
    Apply-then-weight order.  Returns H x W Fractions."""
    H, W = len(U), len(U[0])
    L, k = len(atoms), len(atoms[0])
    r = (k - 1) // 2
    listed = list(range(L)) if kept is None else list(kept)
    scale = [Fr(1)] * len(listed) if gamma is None else list(gamma)
    out = [[Fr(0)] * W for _ in range(H)]
    for Y in range(H):
        for X in range(W):
            total = Fr(0)
            for pos, l in enumerate(listed):
                resp = Fr(0)
                for dy in range(k):
                    for dx in range(k):
                        resp += atoms[l][dy][dx] * U[_clamp(Y + dy - r, 0, H - 1)][_clamp(X + dx - r, 0, W - 1)]
                total += scale[pos] * coeff[l][Y][X] * resp
            out[Y][X] = total
    return out


def to_fractions(a):
    """numpy array (any float dtype) -> nested lists of exact Fractions."""
    if a.ndim == 1:
        return [Fr(float(v)) for v in a]
    return [to_fractions(sub) for sub in a]
