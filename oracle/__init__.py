"""CPU oracle for the dictionary-assembly path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``sr_oracle.c`` (plain C, double precision).  Only
``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg
may import this package; the HIP library and its Python binding never do.

The arithmetic lives in the C file; this module only marshals numpy arrays.
Paper passages followed: section II-A Eq. 2 / Eq. 3 (``F = Phi D``,
``y = F B^T``), section II-B stages 1, 3 and 4, section III-A (atoms with a
zero selector are ignored; kept atoms may be re-scaled).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# The mutation test (tests/test_oracle_mutations.py) points these two at a deliberately
# broken copy of the source to check that the pins notice; nothing else sets them.
_SRC = os.environ.get("SR_ORACLE_SRC") or os.path.join(_HERE, "sr_oracle.c")
_LIB = os.environ.get("SR_ORACLE_LIB") or os.path.join(_HERE, "libsr_oracle.so")

# uint8 arrays are stored 8-bit E4M3 floats, uint16 arrays stored bfloat16 (numpy has no such dtypes)
_DT = {np.dtype(np.float32): 0, np.dtype(np.float16): 1, np.dtype(np.float64): 2, np.dtype(np.uint8): 3,
       np.dtype(np.uint16): 4}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over rows).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_int, c_dbl, c_vp = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        lib.orc_half_to_double.restype = c_dbl
        lib.orc_half_to_double.argtypes = [ctypes.c_uint16]
        lib.orc_e4m3_to_double.restype = c_dbl
        lib.orc_e4m3_to_double.argtypes = [ctypes.c_uint8]
        lib.orc_bf16_to_double.restype = c_dbl
        lib.orc_bf16_to_double.argtypes = [ctypes.c_uint16]
        lib.orc_keys.restype = c_dbl
        lib.orc_keys.argtypes = [c_dbl, c_dbl]
        lib.orc_taps.restype = None
        lib.orc_taps.argtypes = [ctypes.c_long, c_int, c_dbl,
                                 ctypes.POINTER(ctypes.c_long), ctypes.POINTER(c_dbl)]
        lib.orc_bicubic.restype = c_int
        lib.orc_bicubic.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_dbl, c_vp]
        lib.orc_assemble_rows.restype = c_int
        lib.orc_assemble_rows.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp, c_int, c_int,
                                          c_vp, c_int, c_vp, c_int, c_vp, c_int, c_int, c_vp]
        lib.orc_assemble_points.restype = c_int
        lib.orc_assemble_points.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp, c_int, c_int,
                                            c_vp, c_int, c_vp, c_int, c_vp, c_vp, c_int, c_vp]
        lib.orc_assemble_topk_rows.restype = c_int
        lib.orc_assemble_topk_rows.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp, c_int, c_int, c_int,
                                               c_vp, c_int, c_int, c_int, c_vp]
        lib.orc_pixel_major_to_planar.restype = c_int
        lib.orc_pixel_major_to_planar.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_vp]
        lib.orc_blocked_to_planar.restype = c_int
        lib.orc_blocked_to_planar.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_vp]
        lib.orc_pixel_shuffle.restype = c_int
        lib.orc_pixel_shuffle.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_vp]
        lib.orc_round_to_half.restype = c_dbl
        lib.orc_round_to_half.argtypes = [c_dbl]
        lib.orc_softmax_planes.restype = c_int
        lib.orc_softmax_planes.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_vp]
        lib.orc_threads.restype = c_int
        lib.orc_set_threads.restype = c_int
        lib.orc_set_threads.argtypes = [c_int]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _stored(a, name):
    """The caller's stored bytes, untouched: fp16/fp32/fp64, C-contiguous."""
    a = np.asarray(a)
    if a.dtype not in _DT:
        raise TypeError(f"{name}: dtype {a.dtype} not one of float16/32/64, uint8 (= stored E4M3) or uint16 (= stored bfloat16)")
    return np.ascontiguousarray(a)


def half_to_double(bits: int) -> float:
    return _load().orc_half_to_double(int(bits) & 0xFFFF)


def e4m3_to_double(bits: int) -> float:
    return _load().orc_e4m3_to_double(int(bits) & 0xFF)


def bf16_to_double(bits: int) -> float:
    return _load().orc_bf16_to_double(int(bits) & 0xFFFF)


def keys(t: float, a: float = -0.5) -> float:
    return _load().orc_keys(float(t), float(a))


def taps(index: int, scale: int, a: float = -0.5):
    """(first LR tap index, four weights) for HR index ``index``."""
    first = ctypes.c_long()
    w = (ctypes.c_double * 4)()
    _load().orc_taps(int(index), int(scale), float(a), ctypes.byref(first), w)
    return first.value, [w[i] for i in range(4)]


def threads() -> int:
    return _load().orc_threads()


def set_threads(n: int) -> int:
    """Threads for the row loops from now on (timing only); returns the number in force."""
    return _load().orc_set_threads(int(n))


def bicubic(lr, scale: int, a: float = -0.5) -> np.ndarray:
    """Stage 1: ``lr`` [N][C][h][w] -> float64 [N][C][s*h][s*w]."""
    lr = _stored(lr, "lr")
    if lr.dtype in (np.uint8, np.uint16):
        raise TypeError("lr: stored E4M3 and bfloat16 are coefficient formats only")
    if lr.ndim != 4:
        raise ValueError("lr must be [N][C][h][w]")
    n, c, h, w = lr.shape
    U = np.empty((n, c, scale * h, scale * w), dtype=np.float64)
    rc = _load().orc_bicubic(_ptr(lr), _DT[lr.dtype], n, c, h, w, int(scale), float(a), _ptr(U))
    if rc:
        raise ValueError("orc_bicubic rejected its arguments")
    return U


def _common(U, coeff, dictionary, kept, gamma):
    U = np.ascontiguousarray(U, dtype=np.float64)
    coeff = _stored(coeff, "coeff")
    D = np.ascontiguousarray(np.asarray(dictionary).astype(np.float64))
    if U.ndim != 4 or coeff.ndim != 4 or D.ndim != 3 or D.shape[1] != D.shape[2]:
        raise ValueError("shapes: U [N][C][H][W], coeff [N][L][H][W], dict [L][k][k]")
    n, c, H, W = U.shape
    L, k = D.shape[0], D.shape[1]
    if coeff.shape != (n, L, H, W):
        raise ValueError(f"coeff shape {coeff.shape} != {(n, L, H, W)}")
    kept_a = None if kept is None else np.ascontiguousarray(kept, dtype=np.int32)
    gamma_a = None if gamma is None else np.ascontiguousarray(gamma, dtype=np.float64)
    if gamma_a is not None:
        count = L if kept_a is None else kept_a.size
        if gamma_a.size != count:
            raise ValueError("gamma needs one entry per listed atom")
        if kept_a is None:
            kept_a = np.arange(L, dtype=np.int32)
    n_kept = 0 if kept_a is None else int(kept_a.size)
    return U, coeff, D, kept_a, n_kept, gamma_a, (n, c, H, W, L, k)


def assemble(U, coeff, dictionary, kept=None, gamma=None, rows=None) -> np.ndarray:
    """Stages 3 + 4 on a stage-1 result ``U``.  ``rows=(y0, y1)`` limits the HR
    rows computed (others are left at zero)."""
    U, coeff, D, kept_a, n_kept, gamma_a, (n, c, H, W, L, k) = _common(U, coeff, dictionary, kept, gamma)
    y0, y1 = (0, H) if rows is None else rows
    out = np.zeros((n, c, H, W), dtype=np.float64)
    rc = _load().orc_assemble_rows(_ptr(U), n, c, H, W, _ptr(coeff), _DT[coeff.dtype], L,
                                   _ptr(D), k, _ptr(kept_a), n_kept, _ptr(gamma_a),
                                   int(y0), int(y1), _ptr(out))
    if rc:
        raise ValueError("orc_assemble_rows rejected its arguments")
    return out


def assemble_points(U, coeff, dictionary, pts, kept=None, gamma=None) -> np.ndarray:
    """Stages 3 + 4 at listed pixels ``pts`` = [(image, Y, X), ...] -> [n_pts][C]."""
    U, coeff, D, kept_a, n_kept, gamma_a, (n, c, H, W, L, k) = _common(U, coeff, dictionary, kept, gamma)
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 3)
    out = np.zeros((pts.shape[0], c), dtype=np.float64)
    rc = _load().orc_assemble_points(_ptr(U), n, c, H, W, _ptr(coeff), _DT[coeff.dtype], L,
                                     _ptr(D), k, _ptr(kept_a), n_kept, _ptr(gamma_a),
                                     _ptr(pts), pts.shape[0], _ptr(out))
    if rc:
        raise ValueError("orc_assemble_points rejected its arguments")
    return out


def assemble_topk(U, index, value, dictionary, rows=None) -> np.ndarray:
    """Stages 3 + 4 for coefficients given as per-pixel lists (an extension, not in the paper):
    ``index`` uint8 [N][T][H][W] atom numbers, ``value`` [N][T][H][W] their coefficients."""
    U = np.ascontiguousarray(U, dtype=np.float64)
    index = np.ascontiguousarray(index)
    value = _stored(value, "value")
    D = np.ascontiguousarray(np.asarray(dictionary).astype(np.float64))
    if index.dtype != np.uint8 or U.ndim != 4 or index.ndim != 4 or value.shape != index.shape or D.ndim != 3:
        raise ValueError("shapes: U [N][C][H][W], index uint8 and value [N][T][H][W], dict [L][k][k]")
    n, c, H, W = U.shape
    T = index.shape[1]
    if index.shape != (n, T, H, W):
        raise ValueError(f"index shape {index.shape} != {(n, T, H, W)}")
    y0, y1 = (0, H) if rows is None else rows
    out = np.zeros((n, c, H, W), dtype=np.float64)
    rc = _load().orc_assemble_topk_rows(_ptr(U), n, c, H, W, _ptr(index), _ptr(value), _DT[value.dtype], T, D.shape[0],
                                        _ptr(D), D.shape[1], int(y0), int(y1), _ptr(out))
    if rc:
        raise ValueError("orc_assemble_topk_rows rejected its arguments" if rc == -1 else "an index is not below L")
    return out


def pixel_shuffle(coeff_lr, scale: int) -> np.ndarray:
    """What the pixel-shuffle layer at the end of the coefficient network does to its input
    ``coeff_lr`` [N][L*s*s][h][w]: the same stored elements as [N][L][s*h][s*w]."""
    a = _stored(coeff_lr, "coeff_lr")
    if a.ndim != 4 or a.shape[1] % (scale * scale):
        raise ValueError("coeff_lr must be [N][L*s*s][h][w]")
    n, c, h, w = a.shape
    L = c // (scale * scale)
    out = np.empty((n, L, h * scale, w * scale), dtype=a.dtype)
    if _load().orc_pixel_shuffle(_ptr(a), a.dtype.itemsize, n, L, h, w, int(scale), _ptr(out)):
        raise ValueError("orc_pixel_shuffle rejected its arguments")
    return out


def pixel_major_to_planar(coeff_pm) -> np.ndarray:
    """Coefficients stored pixel-major, ``coeff_pm`` [N][H][W][L] (the L coefficients of a pixel side by
    side), as the planar [N][L][H][W] every other function here reads: the same stored elements."""
    a = _stored(coeff_pm, "coeff_pm")
    if a.ndim != 4:
        raise ValueError("coeff_pm must be [N][H][W][L]")
    n, H, W, L = a.shape
    out = np.empty((n, L, H, W), dtype=a.dtype)
    if _load().orc_pixel_major_to_planar(_ptr(a), a.dtype.itemsize, n, L, H, W, _ptr(out)):
        raise ValueError("orc_pixel_major_to_planar rejected its arguments")
    return out


def blocked_to_planar(coeff_blk) -> np.ndarray:
    """Coefficients stored blocked (an extension: the order in which a matrix-core kernel consumes them; see
    orc_blocked_to_planar), ``coeff_blk`` [N][H][W / 128][128 * L] (a row's units of 128 pixels one after the other), as
    the planar [N][L][H][W]: the same stored elements."""
    a = _stored(coeff_blk, "coeff_blk")
    if a.ndim != 4 or a.shape[3] % 128:
        raise ValueError("coeff_blk must be [N][H][W / 128][128 * L]")
    n, H, units, unit_elems = a.shape
    L, W = unit_elems // 128, units * 128
    out = np.empty((n, L, H, W), dtype=a.dtype)
    if _load().orc_blocked_to_planar(_ptr(a), a.dtype.itemsize, n, int(L), H, W, _ptr(out)):
        raise ValueError("orc_blocked_to_planar rejected its arguments (L % 8 == 0 is needed)")
    return out


def round_to_half(v: float) -> float:
    """``v`` rounded to the nearest binary16 value (ties to even), as a double."""
    return _load().orc_round_to_half(float(v))


def softmax_logits(logits, round_half: bool = True) -> np.ndarray:
    """Coefficients from LOGITS (an extension, not in the paper): per pixel the softmax over the atoms of
    ``logits`` [N][L][H][W] (any stored type) -> float64, same shape.  With ``round_half`` (the reading the
    logits form takes) the exponentials ``exp(z - max)`` are rounded to binary16 before they are summed and
    divided; without it this is the plain softmax."""
    z = _stored(logits, "logits")
    if z.ndim != 4:
        raise ValueError("logits must be [N][L][H][W]")
    n, L, H, W = z.shape
    out = np.empty((n, L, H, W), dtype=np.float64)
    if _load().orc_softmax_planes(_ptr(z), _DT[z.dtype], n, L, H, W, 1 if round_half else 0, _ptr(out)):
        raise ValueError("orc_softmax_planes rejected its arguments")
    return out


def dict_assemble(lr, coeff, dictionary, scale: int, kept=None, gamma=None, a: float = -0.5,
                  pre_shuffle: bool = False, pixel_major: bool = False, logits: bool = False, blocked: bool = False) -> np.ndarray:
    """The whole path: stage 1, then stages 3 + 4.  float64 [N][C][s*h][s*w].  With
    ``pre_shuffle`` the coefficients are what the network holds before its pixel-shuffle
    layer, [N][L*s*s][h][w]: that layer is applied first.  With ``pixel_major`` they are stored
    [N][H][W][L] and are moved to planes first; with ``blocked`` they are stored in the blocked order
    (blocked_to_planar) and are moved to planes first.  With ``logits`` the stored values are logits and the
    coefficients their per-pixel softmax (see softmax_logits)."""
    if blocked:                                      # [N][H][W / 128][128 * L], see blocked_to_planar
        coeff = blocked_to_planar(coeff)
    if pixel_major:
        coeff = pixel_major_to_planar(coeff)
    if pre_shuffle:
        coeff = pixel_shuffle(coeff, scale)
    if logits:
        coeff = softmax_logits(coeff)
    return assemble(bicubic(lr, scale, a), coeff, dictionary, kept, gamma)
