"""Seeded synthetic inputs for the dictionary-assembly path.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark, and holds none of the method's arithmetic: it only draws inputs with
the shapes, dtypes and value distributions of the workloads (the paper's
Table I input sizes and scales, plus the 4K and video cases).  The paper's
benchmark images and trained coefficient network are not available; i.i.d.
uniform pixels and softmax-of-Gaussian coefficients stand in for them, because
the cost and the arithmetic of the path do not depend on image content.

Recipe
  * LR image: i.i.d. uniform [0, 1), NCHW.
  * Dictionary [L][k][k] fp32: even atoms are anisotropic rotated Gaussians,
    odd atoms are (1+g)*G(sigma_a) - g*G(sigma_b) with g in [0.5, 2]; every
    Gaussian is sum-normalised on the k x k support and the atom is divided by
    its sum, so each atom sums to 1.
  * Coefficients [N][L][H][W]: per-pixel softmax over the L atoms of Gaussian
    logits, computed in fp32 and then cast to the storage dtype.  "N(m, v)" in
    the workload list is read as mean m, variance v.
  * Logits form: the same Gaussian draws stored as they are (no softmax), cast to the
    storage dtype.
  * Selective workload: a seeded set of 8 dominant atoms has logits N(4, 1) at
    every pixel, the rest N(0, 1).  The kept list is the 8 atoms with the
    largest mean coefficient over the frame (ties go to the lower index).

Everything is drawn with torch generators on the requested device in fixed
row chunks, so a given (config, device type) always yields the same bytes.
Both sides of a parity test consume the same stored bytes.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

BASE_SEED = 230308999
_CHUNK_ROWS = 64  # fixed: changing it changes the drawn bytes


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int           # position in the workload list (seed offset)
    n: int
    c: int
    h: int
    w: int
    scale: int
    L: int
    k: int
    coeff_dtype: str     # "f32" | "f16" | "f8" (8-bit E4M3 storage) | "bf16"
    lr_dtype: str        # "f32" | "f16"  (the output has the LR dtype)
    logit_mean: float = 0.0
    logit_var: float = 1.0
    dominant: int = 0    # >0: that many dominant atoms with logits N(4, 1)

    @property
    def H(self):
        return self.h * self.scale

    @property
    def W(self):
        return self.w * self.scale

    @property
    def hr_pixels(self):
        return self.n * self.H * self.W

    def algorithmic_bytes(self, n_read_atoms=None):
        """Bytes per launch that must cross HBM: every read coefficient once,
        the output once, the LR image once."""
        b_c = {"f32": 4, "f16": 2, "f8": 1, "bf16": 2}[self.coeff_dtype]
        b_io = 2 if self.lr_dtype == "f16" else 4
        atoms = self.L if n_read_atoms is None else n_read_atoms
        per_px = atoms * b_c + self.c * b_io + self.c * b_io / (self.scale ** 2)
        return per_px * self.hr_pixels


WORKLOADS = {
    "tiny": Workload("tiny", 0, 1, 1, 64, 64, 2, 72, 5, "f32", "f32"),
    "720p": Workload("720p", 1, 1, 3, 180, 320, 4, 72, 5, "f32", "f32"),
    "1080p_fp16": Workload("1080p_fp16", 2, 1, 3, 360, 640, 3, 72, 5, "f16", "f32", 0.0, 2.0),
    "4k_dense": Workload("4k_dense", 3, 1, 3, 540, 960, 4, 72, 5, "f16", "f32"),
    # the 4K frame with the coefficients stored as 8-bit floats (same seed: the same
    # softmax values, rounded to E4M3 instead of fp16)
    "4k_dense_fp8": Workload("4k_dense_fp8", 3, 1, 3, 540, 960, 4, 72, 5, "f8", "f32"),
    # ... and as bfloat16 (what a network running in bfloat16 hands over)
    "4k_dense_bf16": Workload("4k_dense_bf16", 3, 1, 3, 540, 960, 4, 72, 5, "bf16", "f32"),
    "4k_selective": Workload("4k_selective", 3, 1, 3, 540, 960, 4, 72, 5, "f16", "f32", 0.0, 1.0, 8),
    "video": Workload("video", 4, 16, 3, 270, 480, 4, 128, 7, "f16", "f16"),
    # beyond the stated list: 1080p x4, whose 72 fp16 planes (4.8 GB) exceed 32-bit byte offsets
    "8k_dense": Workload("8k_dense", 5, 1, 3, 1080, 1920, 4, 72, 5, "f16", "f32"),
}


def to_pre_shuffle(coeff, scale: int):
    """The same stored coefficients in the layout they have before the coefficient network's
    pixel-shuffle layer: [N][L][s*h][s*w] -> [N][L*s*s][h][w] (a move of elements, the inverse of
    that layer; 8-bit floats are moved as bytes)."""
    raw = coeff.view(torch.uint8) if coeff.dtype == torch.float8_e4m3fn else coeff
    pre = torch.nn.functional.pixel_unshuffle(raw, scale).contiguous()
    return pre.view(coeff.dtype) if raw is not coeff else pre


def to_pixel_major(coeff):
    """The same stored coefficients with the L coefficients of a pixel side by side:
    [N][L][H][W] -> [N][H][W][L] (a move of elements; 8-bit floats are moved as bytes)."""
    raw = coeff.view(torch.uint8) if coeff.dtype == torch.float8_e4m3fn else coeff
    pm = raw.permute(0, 2, 3, 1).contiguous()
    return pm.view(coeff.dtype) if raw is not coeff else pm


def to_blocked(coeff):
    """The same stored coefficients in the blocked order (the order in which a matrix-core kernel consumes them; an
    extension of the storage formats): [N][L][H][W] -> [N][H][W / 128][128 * L] with, per row, units of 128 pixels, per unit four
    slots q (pixel 4 j + q is slot q, column j), per slot pieces of 16 atoms [half][j][8 atoms] and, if L % 16 == 8, a
    last piece [half][j][4 atoms].  A move of elements; needs L % 8 == 0 and W % 128 == 0."""
    raw = coeff.view(torch.uint8) if coeff.dtype == torch.float8_e4m3fn else coeff
    n, L, H, W = raw.shape
    assert L % 8 == 0 and W % 128 == 0
    full, units = L // 16, W // 128
    x = raw.reshape(n, L, H, units, 32, 4)                                   # [b][l][y][unit][j][q]
    parts = []
    if full:
        parts.append(x[:, :16 * full].reshape(n, full, 2, 8, H, units, 32, 4)
                     .permute(0, 4, 5, 7, 1, 2, 6, 3).reshape(n, H, units, 4, full * 512))
    if L % 16:
        parts.append(x[:, 16 * full:].reshape(n, 2, 4, H, units, 32, 4)
                     .permute(0, 3, 4, 6, 1, 5, 2).reshape(n, H, units, 4, 256))
    blk = torch.cat(parts, dim=4).reshape(n, H, units, 128 * L).contiguous()
    return blk.view(coeff.dtype) if raw is not coeff else blk


def to_list(coeff, entries: int):
    """The ``entries`` largest coefficients of every pixel as (atom index uint8, value) planes,
    [N][entries][H][W] each, largest first (ties: whatever order the library sort gives; both sides
    of a parity test read the same stored lists).  Values keep the dtype of ``coeff`` (8-bit and
    bfloat16 coefficients are widened to fp16: the list format stores fp16 or fp32 values)."""
    wide = coeff.float() if coeff.dtype in (torch.float16, torch.bfloat16, torch.float8_e4m3fn) else coeff
    val, idx = torch.topk(wide, entries, dim=1)
    vdt = torch.float32 if coeff.dtype == torch.float32 else torch.float16
    return idx.to(torch.uint8).contiguous(), val.to(vdt).contiguous()


def scaled(wl: Workload, **kw) -> Workload:
    """A copy of ``wl`` with some fields replaced (for small test cases)."""
    return dataclasses.replace(wl, **kw)


def torch_dtype(code: str):
    return {"f32": torch.float32, "f16": torch.float16, "f8": torch.float8_e4m3fn, "bf16": torch.bfloat16}[code]


def stored_numpy(t):
    """The stored bytes of a tensor as a numpy array on the host: fp16/fp32 as they are,
    8-bit E4M3 floats as uint8 and bfloat16 as uint16 (numpy has no such dtypes)."""
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).cpu().numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _seed(wl: Workload, stream: int) -> int:
    return (BASE_SEED + wl.index) * 8 + stream


def make_lr(wl: Workload, device="cpu") -> torch.Tensor:
    g = _gen(device, _seed(wl, 0))
    x = torch.rand((wl.n, wl.c, wl.h, wl.w), generator=g, device=device, dtype=torch.float32)
    return x.to(torch_dtype(wl.lr_dtype)).contiguous()


def _gauss(k, sx, sy, theta):
    r = (k - 1) / 2.0
    yy, xx = np.mgrid[0:k, 0:k].astype(np.float64)
    yy -= r
    xx -= r
    ct, st = math.cos(theta), math.sin(theta)
    u = ct * xx + st * yy
    v = -st * xx + ct * yy
    g = np.exp(-0.5 * ((u / sx) ** 2 + (v / sy) ** 2))
    return g / g.sum()


def make_dictionary(wl: Workload, device="cpu") -> torch.Tensor:
    """[L][k][k] fp32 Gaussian / difference-of-Gaussians atoms, each summing to 1."""
    rng = np.random.Generator(np.random.PCG64(_seed(wl, 1)))
    smax = 2.5 if wl.k <= 5 else 3.5
    atoms = np.empty((wl.L, wl.k, wl.k), dtype=np.float64)
    for l in range(wl.L):
        if l % 2 == 0:
            sx, sy = rng.uniform(0.5, smax, size=2)
            atom = _gauss(wl.k, sx, sy, rng.uniform(0.0, math.pi))
        else:
            sa, sb = np.sort(rng.uniform(0.5, smax, size=2))
            gain = rng.uniform(0.5, 2.0)
            th = rng.uniform(0.0, math.pi)
            atom = (1.0 + gain) * _gauss(wl.k, sa, sa * rng.uniform(0.7, 1.0), th) \
                - gain * _gauss(wl.k, sb + 0.25, sb + 0.25, 0.0)
        atoms[l] = atom / atom.sum()
    return torch.from_numpy(atoms.astype(np.float32)).to(device).contiguous()


def dominant_atoms(wl: Workload) -> np.ndarray:
    """The seeded set of dominant atoms of a selective workload (sorted)."""
    rng = np.random.Generator(np.random.PCG64(_seed(wl, 3)))
    return np.sort(rng.choice(wl.L, size=wl.dominant, replace=False)).astype(np.int32)


def make_coeff(wl: Workload, device="cpu", return_mean=False):
    """[N][L][H][W] coefficients in the storage dtype; optionally also the
    per-atom mean of the stored values (float64 numpy, length L)."""
    dt = torch_dtype(wl.coeff_dtype)
    H, W = wl.H, wl.W
    out = torch.empty((wl.n, wl.L, H, W), device=device, dtype=dt)
    g = _gen(device, _seed(wl, 2))
    std = math.sqrt(wl.logit_var)
    shift = None
    if wl.dominant:
        shift = torch.zeros((wl.L, 1, 1), device=device, dtype=torch.float32)
        shift[torch.from_numpy(dominant_atoms(wl).astype(np.int64)).to(device)] = 4.0
    total = torch.zeros(wl.L, device=device, dtype=torch.float64)
    for b in range(wl.n):
        for y0 in range(0, H, _CHUNK_ROWS):
            rows = min(_CHUNK_ROWS, H - y0)
            logits = torch.randn((wl.L, rows, W), generator=g, device=device, dtype=torch.float32)
            logits = logits * std + wl.logit_mean
            if shift is not None:
                logits = logits + shift
            chunk = torch.softmax(logits, dim=0).to(dt)
            out[b, :, y0:y0 + rows, :] = chunk
            if return_mean:
                total += chunk.to(torch.float64).sum(dim=(1, 2))
    if return_mean:
        return out, (total / float(wl.n * H * W)).cpu().numpy()
    return out


def make_logits(wl: Workload, device="cpu"):
    """[N][L][H][W] LOGITS in the storage dtype: the Gaussian draws of ``make_coeff`` (same seed, same
    order) as they are before its softmax, for the path's logits form."""
    dt = torch_dtype(wl.coeff_dtype)
    H, W = wl.H, wl.W
    out = torch.empty((wl.n, wl.L, H, W), device=device, dtype=dt)
    g = _gen(device, _seed(wl, 2))
    std = math.sqrt(wl.logit_var)
    shift = None
    if wl.dominant:
        shift = torch.zeros((wl.L, 1, 1), device=device, dtype=torch.float32)
        shift[torch.from_numpy(dominant_atoms(wl).astype(np.int64)).to(device)] = 4.0
    for b in range(wl.n):
        for y0 in range(0, H, _CHUNK_ROWS):
            rows = min(_CHUNK_ROWS, H - y0)
            logits = torch.randn((wl.L, rows, W), generator=g, device=device, dtype=torch.float32)
            logits = logits * std + wl.logit_mean
            if shift is not None:
                logits = logits + shift
            out[b, :, y0:y0 + rows, :] = logits.to(dt)
    return out


def kept_from_mean(mean: np.ndarray, count: int) -> np.ndarray:
    """Indices of the ``count`` largest means, ties to the lower index, ascending."""
    order = sorted(range(len(mean)), key=lambda i: (-float(mean[i]), i))
    return np.array(sorted(order[:count]), dtype=np.int32)


def make_inputs(wl: Workload, device="cpu"):
    """dict(lr, coeff, dict[, kept]) of torch tensors on ``device`` (kept: numpy int32)."""
    res = {"lr": make_lr(wl, device), "dict": make_dictionary(wl, device)}
    if wl.dominant:
        coeff, mean = make_coeff(wl, device, return_mean=True)
        res["coeff"] = coeff
        res["kept"] = kept_from_mean(mean, wl.dominant)
    else:
        res["coeff"] = make_coeff(wl, device)
    return res
