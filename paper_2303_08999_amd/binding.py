"""ctypes binding of libsrdict.so: argument marshalling only.

Each function has the name and argument order of the C entry point declared in
include/sr_dict.h and takes torch tensors living in device memory; every step
of the path runs inside the library's HIP kernels.  There is no CPU fallback:
if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsrdict.so")

SR_F32, SR_F16, SR_F8E4M3, SR_BF16, SR_U8 = 0, 1, 2, 3, 4
SR_KERNEL_AUTO, SR_KERNEL_GENERIC, SR_KERNEL_MFMA = 0, 1, 2
SR_COEFF_PLANAR, SR_COEFF_PRE_SHUFFLE, SR_COEFF_PIXEL_MAJOR, SR_COEFF_BLOCKED = 0, 1, 2, 3
SR_COEFF_VALUES, SR_COEFF_LOGITS = 0, 1
SR_MAX_ATOMS = 256

EXPORTS = ("sr_dict_assemble", "sr_dict_assemble_selective", "sr_dict_assemble_ex", "sr_dict_assemble_list", "sr_dict_assemble_list_ex",
           "sr_bicubic_upsample", "sr_dict_assemble_plan", "sr_dict_assemble_tile", "sr_dict_assemble_launch_shape", "sr_strerror", "sr_version",
           "sr_probe_read", "sr_probe_mix", "sr_probe_mix_tiled", "sr_probe_mix_tiled_bytes", "sr_probe_mix_tiled_paced", "sr_probe_stream", "sr_probe_pattern", "sr_probe_policy", "sr_probe_policy_bits",
           "sr_atom_gram_workspace_bytes", "sr_atom_gram", "sr_atom_gram_static", "sr_select_atoms")


class sr_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int),
                ("n", ctypes.c_int), ("c", ctypes.c_int), ("h", ctypes.c_int), ("w", ctypes.c_int)]


class sr_options(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int), ("tile", ctypes.c_int), ("coeff_layout", ctypes.c_int),
                ("coeff_kind", ctypes.c_int), ("reserved", ctypes.c_int * 4)]


class SrError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"libsrdict status {status}: {text}")
        self.status = status


_lib = None


def load():
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first with __graft_entry__.build() "
            "(python -m paper_2303_08999_amd.build); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    T, O = ctypes.POINTER(sr_tensor), ctypes.POINTER(sr_options)
    i, vp = ctypes.c_int, ctypes.c_void_p
    ip, fp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)
    lib.sr_dict_assemble.argtypes = [T, T, T, i, i, i, i, T, vp]
    lib.sr_dict_assemble_selective.argtypes = [T, T, T, i, i, i, i, T, vp, ip, i, fp]
    lib.sr_dict_assemble_ex.argtypes = [T, T, T, i, i, i, i, T, vp, ip, i, fp, O]
    lib.sr_dict_assemble_list.argtypes = [T, T, T, T, i, i, i, i, i, T, vp]
    lib.sr_dict_assemble_list_ex.argtypes = [T, T, T, T, i, i, i, i, i, T, vp, i]
    lib.sr_dict_assemble_plan.argtypes = [T, T, T, i, i, i, i, T, ip, i, O]
    lib.sr_dict_assemble_tile.argtypes = [T, T, T, i, i, i, i, T, ip, i, O, ip, ip]
    lib.sr_dict_assemble_launch_shape.argtypes = [T, T, T, i, i, i, i, T, ip, i, O, ip]
    lib.sr_dict_assemble_launch_shape.restype = i
    lib.sr_bicubic_upsample.argtypes = [T, i, i, T, vp]
    lib.sr_strerror.argtypes = [i]
    lib.sr_probe_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.sr_probe_mix.argtypes = [vp, i, ctypes.c_size_t, vp, i, vp]
    lib.sr_probe_mix_tiled.argtypes = [vp, i, i, i, i, vp, i, vp]
    lib.sr_probe_mix_tiled.restype = i
    lib.sr_probe_mix_tiled_bytes.argtypes = [vp, i, i, i, i, i, vp, i, vp]
    lib.sr_probe_mix_tiled_bytes.restype = i
    lib.sr_probe_mix_tiled_paced.argtypes = [vp, i, i, i, i, i, vp, i, i, vp]
    lib.sr_probe_mix_tiled_paced.restype = i
    lib.sr_probe_pattern.argtypes = [vp, vp, ctypes.c_size_t, i, i, i, i, i, ctypes.c_size_t, vp, vp]
    lib.sr_probe_policy.argtypes = [vp, vp, ctypes.c_size_t, i, i, i, i, vp, vp]
    lib.sr_probe_policy_bits.argtypes = [vp, vp, ctypes.c_size_t, i, i, i, vp, vp]
    lib.sr_probe_stream.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, i, i, i, i, vp, vp]
    dp = ctypes.POINTER(ctypes.c_double)
    lib.sr_atom_gram_workspace_bytes.argtypes = [i]
    lib.sr_atom_gram.argtypes = [T, T, T, T, i, i, i, i, vp, ctypes.c_size_t, vp, vp]
    lib.sr_atom_gram_static.argtypes = [T, T, T, T, i, i, i, i, vp, vp]
    lib.sr_select_atoms.argtypes = [dp, i, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                    ip, ip, fp, dp]
    lib.sr_strerror.restype = ctypes.c_char_p
    lib.sr_version.argtypes = []
    for name in EXPORTS:
        if name not in ("sr_strerror", "sr_atom_gram_workspace_bytes"):
            getattr(lib, name).restype = i
    lib.sr_atom_gram_workspace_bytes.restype = ctypes.c_size_t
    _lib = lib
    return lib


def describe(t) -> sr_tensor:
    """sr_tensor descriptor of a contiguous 4-D torch tensor (no copy)."""
    import torch
    if t.dim() != 4 or not t.is_contiguous():
        raise ValueError("expected a contiguous [N][C][H][W] tensor")
    if t.dtype == torch.float32:
        code = SR_F32
    elif t.dtype == torch.float16:
        code = SR_F16
    elif t.dtype == torch.float8_e4m3fn:
        code = SR_F8E4M3
    elif t.dtype == torch.bfloat16:
        code = SR_BF16
    elif t.dtype == torch.uint8:
        code = SR_U8
    else:
        raise TypeError(f"dtype {t.dtype} is not float32/float16/float8_e4m3fn/bfloat16")
    ptr = t.data_ptr() if t.numel() else 0
    return sr_tensor(ptr or None, code, *[int(v) for v in t.shape])


def describe_coeff(t, opts=None) -> sr_tensor:
    """Descriptor of the coefficient tensor for the layout named in ``opts``: a pixel-major tensor
    [N][H][W][L] is described with c = L, h = H, w = W, as the header asks, and so is a blocked one."""
    d = describe(t)
    if opts is not None and opts.coeff_layout == SR_COEFF_PIXEL_MAJOR:
        d.c, d.h, d.w = int(t.shape[3]), int(t.shape[1]), int(t.shape[2])
    if opts is not None and opts.coeff_layout == SR_COEFF_BLOCKED:           # [N][H][W / 128][128 * L]
        d.c, d.h, d.w = int(t.shape[3]) // 128, int(t.shape[1]), int(t.shape[2]) * 128
    return d


def _dict4(d):
    return d if d.dim() == 4 else d.reshape(1, *d.shape)


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status):
    if status != 0:
        raise SrError(status, sr_strerror(status))


def _host_lists(kept, gamma):
    if kept is None:
        return None, 0, None, ()
    kept = [int(v) for v in kept]
    ka = (ctypes.c_int * max(1, len(kept)))(*kept)
    ga = None
    if gamma is not None:
        gamma = [float(v) for v in gamma]
        if len(gamma) != len(kept):
            raise ValueError("gamma needs one entry per kept atom")
        ga = (ctypes.c_float * max(1, len(gamma)))(*gamma)
    return ka, len(kept), ga, (ka, ga)


def sr_strerror(status: int) -> str:
    return load().sr_strerror(int(status)).decode()


def sr_version() -> int:
    return load().sr_version()


def sr_dict_assemble(lr, coeff, dict, L, k, scale, channels, out, stream=None):
    a, b, c, o = describe(lr), describe(coeff), describe(_dict4(dict)), describe(out)
    _check(load().sr_dict_assemble(a, b, c, L, k, scale, channels, o, _stream(stream)))
    return out


def sr_dict_assemble_selective(lr, coeff, dict, L, k, scale, channels, out, stream=None,
                               kept=None, n_kept=None, gamma=None):
    a, b, c, o = describe(lr), describe(coeff), describe(_dict4(dict)), describe(out)
    ka, n, ga, _keep = _host_lists(kept, gamma)
    n = n if n_kept is None else int(n_kept)
    _check(load().sr_dict_assemble_selective(a, b, c, L, k, scale, channels, o, _stream(stream), ka, n, ga))
    return out


def make_options(kernel=SR_KERNEL_AUTO, tile=0, coeff_layout=SR_COEFF_PLANAR, coeff_kind=SR_COEFF_VALUES) -> sr_options:
    o = sr_options()
    o.kernel, o.tile, o.coeff_layout, o.coeff_kind = int(kernel), int(tile), int(coeff_layout), int(coeff_kind)
    return o


def sr_dict_assemble_ex(lr, coeff, dict, L, k, scale, channels, out, stream=None,
                        kept=None, n_kept=None, gamma=None, opts=None):
    a, b, c, o = describe(lr), describe_coeff(coeff, opts), describe(_dict4(dict)), describe(out)
    ka, n, ga, _keep = _host_lists(kept, gamma)
    n = n if n_kept is None else int(n_kept)
    op = ctypes.byref(opts) if opts is not None else None
    _check(load().sr_dict_assemble_ex(a, b, c, L, k, scale, channels, o, _stream(stream), ka, n, ga, op))
    return out


def sr_dict_assemble_plan(lr, coeff, dict, L, k, scale, channels, out, kept=None, n_kept=None, opts=None) -> int:
    a, b, c, o = describe(lr), describe_coeff(coeff, opts), describe(_dict4(dict)), describe(out)
    ka, n, _ga, _keep = _host_lists(kept, None)
    n = n if n_kept is None else int(n_kept)
    op = ctypes.byref(opts) if opts is not None else None
    return load().sr_dict_assemble_plan(a, b, c, L, k, scale, channels, o, ka, n, op)


def sr_dict_assemble_list(lr, index, value, dict, L, k, scale, channels, entries, out, stream=None):
    """Coefficients as per-pixel (atom index, value) lists, an extension beyond the paper (include/sr_dict.h)."""
    _check(load().sr_dict_assemble_list(describe(lr), describe(index), describe(value), describe(_dict4(dict)),
                                        L, k, scale, channels, entries, describe(out), _stream(stream)))
    return out


def sr_dict_assemble_list_ex(lr, index, value, dict, L, k, scale, channels, entries, out, stream=None,
                             kernel=SR_KERNEL_AUTO):
    _check(load().sr_dict_assemble_list_ex(describe(lr), describe(index), describe(value), describe(_dict4(dict)),
                                           L, k, scale, channels, entries, describe(out), _stream(stream), int(kernel)))
    return out


def sr_dict_assemble_tile(lr, coeff, dict, L, k, scale, channels, out, kept=None, n_kept=None, opts=None):
    """(kernel or negative status, tile width, tile height) the call would run with."""
    a, b, c, o = describe(lr), describe_coeff(coeff, opts), describe(_dict4(dict)), describe(out)
    ka, n, _ga, _keep = _host_lists(kept, None)
    n = n if n_kept is None else int(n_kept)
    op = ctypes.byref(opts) if opts is not None else None
    tw, th = ctypes.c_int(0), ctypes.c_int(0)
    st = load().sr_dict_assemble_tile(a, b, c, L, k, scale, channels, o, ka, n, op, ctypes.byref(tw), ctypes.byref(th))
    return st, tw.value, th.value


def sr_dict_assemble_launch_shape(lr, coeff, dict, L, k, scale, channels, out, kept=None, n_kept=None, opts=None):
    """(kernel or negative status, (tile width, tile height, wavefronts per workgroup, workgroups per CU))."""
    a, b, c, o = describe(lr), describe_coeff(coeff, opts), describe(_dict4(dict)), describe(out)
    ka, n, _ga, _keep = _host_lists(kept, None)
    n = n if n_kept is None else int(n_kept)
    op = ctypes.byref(opts) if opts is not None else None
    shape = (ctypes.c_int * 4)()
    st = load().sr_dict_assemble_launch_shape(a, b, c, L, k, scale, channels, o, ka, n, op, shape)
    return st, tuple(shape)


def sr_bicubic_upsample(lr, scale, channels, out, stream=None):
    _check(load().sr_bicubic_upsample(describe(lr), scale, channels, describe(out), _stream(stream)))
    return out


def sr_probe_read(src, sink, stream=None):
    """Streaming read of the whole tensor ``src`` (include/sr_probe.h); ``sink`` is any
    device tensor of at least 4 bytes."""
    nbytes = src.numel() * src.element_size()
    _check(load().sr_probe_read(ctypes.c_void_p(src.data_ptr()), nbytes,
                                ctypes.c_void_p(sink.data_ptr()), _stream(stream)))


def sr_probe_mix(coeff, planes, pixels, out, channels, stream=None):
    """The assembly kernel's read + write stream with no work in it (include/sr_probe.h)."""
    assert coeff.numel() * coeff.element_size() >= planes * pixels * 2
    assert out.numel() * out.element_size() >= channels * pixels * 4
    _check(load().sr_probe_mix(ctypes.c_void_p(coeff.data_ptr()), planes, pixels,
                               ctypes.c_void_p(out.data_ptr()), channels, _stream(stream)))


def sr_probe_mix_tiled(coeff, planes, height, width, tile_h, out, channels, stream=None, elem_bytes=2, pace_us=0):
    """The assembly kernel's memory requests in its own tile order, nothing else (include/sr_probe.h);
    ``elem_bytes`` = 1 for planes of 8-bit coefficients (sr_probe_mix_tiled_bytes); ``pace_us`` > 0 adds the kernel's
    L2 write-back pacing (sr_probe_mix_tiled_paced)."""
    assert coeff.numel() * coeff.element_size() >= planes * height * width * elem_bytes
    assert out.numel() * out.element_size() >= channels * height * width * 4
    if pace_us:
        _check(load().sr_probe_mix_tiled_paced(ctypes.c_void_p(coeff.data_ptr()), planes, elem_bytes, height, width, tile_h,
                                               ctypes.c_void_p(out.data_ptr()), channels, int(pace_us), _stream(stream)))
    elif elem_bytes == 2:
        _check(load().sr_probe_mix_tiled(ctypes.c_void_p(coeff.data_ptr()), planes, height, width, tile_h,
                                         ctypes.c_void_p(out.data_ptr()), channels, _stream(stream)))
    else:
        _check(load().sr_probe_mix_tiled_bytes(ctypes.c_void_p(coeff.data_ptr()), planes, elem_bytes, height, width, tile_h,
                                               ctypes.c_void_p(out.data_ptr()), channels, _stream(stream)))


def sr_probe_stream(src, read_bytes, dst, write_bytes, blocks, writer_every, sink, lds_bytes=0, nt_store=0, stream=None):
    """Readers and writers in separate workgroups, 16 bytes per lane (include/sr_probe.h)."""
    assert src is None or src.numel() * src.element_size() >= read_bytes
    assert dst is None or dst.numel() * dst.element_size() >= write_bytes
    _check(load().sr_probe_stream(ctypes.c_void_p(src.data_ptr() if src is not None else 0), read_bytes,
                                  ctypes.c_void_p(dst.data_ptr() if dst is not None else 0), write_bytes,
                                  blocks, writer_every, lds_bytes, nt_store,
                                  ctypes.c_void_p(sink.data_ptr()), _stream(stream)))


def sr_probe_pattern(src, dst, pixels, read_planes, write_planes, same_wave, blocks, writer_every, sink,
                     plane_pad_bytes=0, stream=None):
    """72 fp16 planes read, 3 fp32 planes written, one pattern property at a time (include/sr_probe.h)."""
    assert src.numel() * src.element_size() >= 72 * (2 * pixels + plane_pad_bytes)
    assert dst.numel() * dst.element_size() >= 12 * pixels
    _check(load().sr_probe_pattern(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), pixels,
                                   int(read_planes), int(write_planes), int(same_wave), blocks, writer_every,
                                   plane_pad_bytes,
                                   ctypes.c_void_p(sink.data_ptr()), _stream(stream)))


def sr_probe_policy(src, dst, pixels, load_policy, store_policy, flush_every, blocks, sink, stream=None):
    """The assembly kernel's byte mix under other cache policies (include/sr_probe.h)."""
    assert src.numel() * src.element_size() >= 144 * pixels and dst.numel() * dst.element_size() >= 12 * pixels
    _check(load().sr_probe_policy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), pixels,
                                  load_policy, store_policy, flush_every, blocks,
                                  ctypes.c_void_p(sink.data_ptr()), _stream(stream)))


def sr_probe_policy_bits(src, dst, pixels, load_bits, store_bits, blocks, sink, stream=None):
    """The assembly kernel's byte mix under any cache-policy bits, sc0 | sc1 << 1 | nt << 2 (include/sr_probe.h)."""
    assert src.numel() * src.element_size() >= 144 * pixels and dst.numel() * dst.element_size() >= 12 * pixels
    _check(load().sr_probe_policy_bits(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), pixels,
                                       load_bits, store_bits, blocks, ctypes.c_void_p(sink.data_ptr()), _stream(stream)))


def sr_atom_gram_workspace_bytes(L: int) -> int:
    return int(load().sr_atom_gram_workspace_bytes(int(L)))


def sr_atom_gram(up, coeff, dict, target, L, k, channels, stride=1, workspace=None, normal=None, stream=None):
    """Normal equations of the selection regression (include/sr_select.h).  Returns the
    device tensor of L*L + L + 2 doubles (G, b, hh, M); scratch and result are torch
    tensors made here unless the caller passes them."""
    import torch
    need = sr_atom_gram_workspace_bytes(L)
    if workspace is None:
        workspace = torch.empty(max(need, 16), device=up.device, dtype=torch.uint8)
    if normal is None:
        normal = torch.empty(L * L + L + 2, device=up.device, dtype=torch.float64)
    _check(load().sr_atom_gram(describe(up), describe(coeff), describe(_dict4(dict)), describe(target),
                               L, k, channels, stride, ctypes.c_void_p(workspace.data_ptr()),
                               workspace.numel() * workspace.element_size(),
                               ctypes.c_void_p(normal.data_ptr()), _stream(stream)))
    return normal


def sr_atom_gram_static(up, coeff, dict, target, L, k, channels, stride, normal, stream=None):
    """sr_atom_gram on the library's built-in scratch (include/sr_select.h).  Nothing is allocated,
    here or in the library: `normal` (L*L + L + 2 float64 on the device) is the caller's."""
    _check(load().sr_atom_gram_static(describe(up), describe(coeff), describe(_dict4(dict)), describe(target),
                                      L, k, channels, stride, ctypes.c_void_p(normal.data_ptr()), _stream(stream)))
    return normal


def sr_select_atoms(normal, L, alpha, delta_alpha=0.1, lambda0=1e-6, eps=0.0):
    """Alg. 1 on host normal equations (a numpy float64 array of L*L + L + 2 values).
    Returns (kept indices int32 ascending, gamma float32, lambda reached)."""
    import numpy as np
    nm = np.ascontiguousarray(normal, dtype=np.float64)
    if nm.size != L * L + L + 2:
        raise ValueError("normal must hold L*L + L + 2 values")
    kept = np.zeros(L, dtype=np.int32)
    gamma = np.zeros(L, dtype=np.float32)
    n = ctypes.c_int(0)
    lam = ctypes.c_double(0.0)
    _check(load().sr_select_atoms(nm.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), L, alpha, delta_alpha,
                                  lambda0, eps, kept.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), ctypes.byref(n),
                                  gamma.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), ctypes.byref(lam)))
    return kept[:n.value].copy(), gamma[:n.value].copy(), lam.value
