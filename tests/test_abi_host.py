"""Host-side checks of the C ABI: the library loads without a GPU, exports every
symbol the header declares, and rejects bad arguments before launching anything.
No compute call is made here."""
import ctypes
import os
import re

import pytest

import paper_2303_08999_amd as sr
from paper_2303_08999_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2303_08999_amd import build
        build.build_library()
    return sr.load()


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if header.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, header)).read(), flags=re.S)
            names.update(re.findall(r"\b(sr_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_a_missing_library_fails_loudly(lib, tmp_path, monkeypatch):
    """There is no fallback path: with no built library the binding raises, it computes nothing another way."""
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libsrdict.so"))
    monkeypatch.setattr(binding, "_lib", None, raising=False)
    with pytest.raises(ImportError, match="is missing"):
        binding.load()


def test_version_and_strerror(lib):
    assert sr.sr_version() == 300
    assert sr.sr_strerror(0) == "success"
    for code in range(-8, 0):
        assert sr.sr_strerror(code) not in ("", "success", "unknown status")
    assert sr.sr_strerror(-99) == "unknown status"


def T(ptr, dtype, n, c, h, w):
    return sr.sr_tensor(ptr, dtype, n, c, h, w)


def case(L=72, k=5, s=4, C=3, h=8, w=16, cd=sr.SR_F16, io=sr.SR_F32, base=0x10000000):
    """Descriptors with fake, well-separated, aligned device addresses."""
    lr = T(base, io, 1, C, h, w)
    coeff = T(base + 0x1000000, cd, 1, L, s * h, s * w)
    d = T(base + 0x8000000, sr.SR_F32, 1, L, k, k)
    out = T(base + 0x9000000, io, 1, C, s * h, s * w)
    return lr, coeff, d, out


def plan(lr, coeff, d, out, L=72, k=5, s=4, C=3, kept=None, opts=None):
    ka = None
    n = 0
    if kept is not None:
        ka = (ctypes.c_int * max(1, len(kept)))(*kept)
        n = len(kept)
    op = ctypes.byref(opts) if opts is not None else None
    return sr.load().sr_dict_assemble_plan(lr, coeff, d, L, k, s, C, out, ka, n, op)


def test_plan_accepts_a_good_case(lib):
    assert plan(*case()) in (sr.SR_KERNEL_GENERIC, sr.SR_KERNEL_MFMA)
    assert plan(*case(cd=sr.SR_F32)) == sr.SR_KERNEL_MFMA           # fp32 coefficients: fp32 MFMA
    assert plan(*case(cd=sr.SR_F32, k=7), k=7) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=sr.SR_F8E4M3, k=7), k=7) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=sr.SR_F8E4M3, k=7, L=16), k=7, L=16) == sr.SR_KERNEL_GENERIC   # short 7x7 lists stay generic
    assert plan(*case(cd=sr.SR_F32, w=15, s=2), s=2) == sr.SR_KERNEL_MFMA   # HR width 30: even is enough
    assert plan(*case(k=3), k=3) == sr.SR_KERNEL_MFMA
    assert plan(*case(k=3, C=2), k=3, C=2) == sr.SR_KERNEL_GENERIC          # two and four channels: 5x5, fp16 coefficients only
    assert plan(*case(C=4), C=4) == sr.SR_KERNEL_MFMA
    assert plan(*case(C=2), C=2) == sr.SR_KERNEL_MFMA
    assert plan(*case(C=5), C=5) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=15, s=3), s=3) == sr.SR_KERNEL_GENERIC   # HR width 45: not whole groups of four pixels and under 128
    assert plan(*case(w=43, s=3), s=3) == sr.SR_KERNEL_MFMA      # HR width 129: the last tile column ends at the image edge
    assert plan(*case(w=1, s=3), s=3) == sr.SR_KERNEL_GENERIC    # HR width 3: not even one group of four pixels
    assert plan(*case(w=15), opts=sr.make_options(sr.SR_KERNEL_MFMA)) == sr.SR_KERNEL_MFMA   # width 60
    assert plan(*case(L=73), L=73) == sr.SR_KERNEL_MFMA          # 73 to 128 atoms of 5x5: fp16 and bfloat16
    assert plan(*case(L=129), L=129) == sr.SR_KERNEL_GENERIC     # more atoms than the 5x5 kernel holds
    assert plan(*case(L=73, cd=sr.SR_F32), L=73) == sr.SR_KERNEL_MFMA
    assert plan(*case(L=128, cd=sr.SR_F8E4M3), L=128) == sr.SR_KERNEL_MFMA
    assert plan(*case(L=73, k=3), L=73, k=3) == sr.SR_KERNEL_MFMA
    assert plan(*case(L=129, k=3), L=129, k=3) == sr.SR_KERNEL_GENERIC
    assert plan(*case(L=128, k=7), L=128, k=7) == sr.SR_KERNEL_MFMA
    assert plan(*case(), opts=sr.make_options(sr.SR_KERNEL_GENERIC)) == sr.SR_KERNEL_GENERIC


def test_plan_for_images_with_more_than_4_gb_of_coefficients(lib):
    """An 8K frame: 72 fp16 planes of 7680 x 4320 are 4.8 GB.  The matrix-core kernel takes it
    with element offsets where such instantiations exist (5x5, three channels, fp16)."""
    def big(L=72, k=5, C=3, cd=sr.SR_F16, h=1080, w=1920, s=4):
        lr = T(0x10000000, sr.SR_F32, 1, C, h, w)
        coeff = T(0x100000000, cd, 1, L, s * h, s * w)
        d = T(0x800000000, sr.SR_F32, 1, L, k, k)
        out = T(0x900000000, sr.SR_F32, 1, C, s * h, s * w)
        return lr, coeff, d, out
    assert plan(*big()) == sr.SR_KERNEL_MFMA
    assert plan(*big(), kept=[1, 5, 71]) == sr.SR_KERNEL_MFMA
    assert plan(*big(cd=sr.SR_F8E4M3)) == sr.SR_KERNEL_MFMA          # 2.4 GB: ordinary byte offsets
    assert plan(*big(cd=sr.SR_BF16)) == sr.SR_KERNEL_MFMA
    assert plan(*big(C=1), C=1) == sr.SR_KERNEL_GENERIC
    assert plan(*big(cd=sr.SR_F32)) == sr.SR_KERNEL_GENERIC
    assert plan(*big(L=128, k=7), L=128, k=7) == sr.SR_KERNEL_GENERIC
    assert plan(*big(h=2160, w=3840)) == sr.SR_KERNEL_GENERIC        # 16K: more than 2^32 coefficients
    assert plan(*big(), opts=sr.make_options(sr.SR_KERNEL_MFMA)) == sr.SR_KERNEL_MFMA
    # the element-offset instantiations hold at most 72 folded atoms: more must not be served by them
    for L in (73, 100, 128):
        assert L * 4320 * 7680 < 2**32 <= 2 * L * 4320 * 7680
        assert plan(*big(L=L), L=L) == sr.SR_KERNEL_GENERIC
        assert plan(*big(L=L, cd=sr.SR_BF16), L=L) == sr.SR_KERNEL_GENERIC
        assert plan(*big(L=L), L=L, opts=sr.make_options(sr.SR_KERNEL_MFMA)) == -3
        assert plan(*big(L=L), L=L, kept=list(range(72))) == sr.SR_KERNEL_MFMA     # a list of 72 of them is fine
        assert plan(*big(L=L), L=L, kept=list(range(73))) == sr.SR_KERNEL_GENERIC


def tile_of(lr, coeff, d, out, L=72, k=5, s=4, C=3, kept=None, opts=None):
    ka, n = None, 0
    if kept is not None:
        ka, n = (ctypes.c_int * max(1, len(kept)))(*kept), len(kept)
    tw, th = ctypes.c_int(-1), ctypes.c_int(-1)
    st = sr.load().sr_dict_assemble_tile(lr, coeff, d, L, k, s, C, out, ka, n,
                                         ctypes.byref(opts) if opts is not None else None, ctypes.byref(tw), ctypes.byref(th))
    return st, tw.value, th.value


def test_tile_indices_name_distinct_instantiations_or_are_refused(lib):
    """The launch-shape option (section III-B): every accepted index is a different tile, and a family
    with one built shape accepts index 0 only - a sweep never times one kernel under several names."""
    MF, AUTO = sr.SR_KERNEL_MFMA, sr.SR_KERNEL_AUTO

    def far(**kw):                                   # the same descriptors, 64 GB apart: room for whole frames
        ts = case(**kw)
        for i, t in enumerate(ts):
            t.data = 0x1000000000 * (i + 1)
        return ts
    shapes = {}
    launch = {}
    for tile in range(0, 12):
        st, tw, th = tile_of(*far(h=540, w=960), opts=sr.make_options(MF, tile))
        ts = far(h=540, w=960)
        shape4 = (ctypes.c_int * 4)()
        st2 = lib.sr_dict_assemble_launch_shape(*ts[:3], 72, 5, 4, 3, ts[3], None, 0, ctypes.byref(sr.make_options(MF, tile)), shape4)
        if tile <= 9:
            assert st == MF and tw > 0 and th > 0, (tile, st)
            shapes[tile] = (tw, th)
            assert st2 == MF and tuple(shape4)[:2] == (tw, th) and shape4[2] in (2, 4, 8) and shape4[3] in (1, 2)
            launch[tile] = tuple(shape4)
        else:
            assert st == -3 and st2 == -3
    assert len({shapes[t] for t in range(1, 8)}) == 7                      # seven different tiles
    assert shapes[0] == shapes[7] == (128, 24)                              # the 4K frame's default
    assert len({launch[t] for t in range(1, 10)}) == 9                     # nine different launch shapes
    assert launch[6] == (128, 16, 4, 2) and launch[8] == (128, 16, 8, 1) and launch[9] == (128, 16, 2, 2)
    assert lib.sr_dict_assemble_launch_shape(*far(h=540, w=960)[:3], 72, 5, 4, 3, far(h=540, w=960)[3], None, 0, None, None) == -1
    assert tile_of(*far(h=64, w=64), opts=sr.make_options(MF, 0))[1:] == (128, 4)       # small frame
    assert tile_of(*far(h=270, w=480), opts=sr.make_options(MF, 0))[1:] == (64, 16)     # 1080p at x4
    assert tile_of(*far(h=360, w=640, s=3), s=3, opts=sr.make_options(MF, 0))[1:] == (128, 16)
    assert tile_of(*far(h=360, w=640, s=3), s=3, opts=sr.make_options(MF, 7))[0] == -3  # 128 x 24 needs scale 4
    # families without alternatives: index 0 only, under AUTO as well (no silent fall-back to another kernel)
    for kw, pk in (({"cd": sr.SR_F32}, {}), ({"cd": sr.SR_F8E4M3}, {}), ({"cd": sr.SR_BF16}, {}), ({"k": 7}, {"k": 7}),
                   ({"k": 3}, {"k": 3}), ({"C": 1}, {"C": 1}), ({"L": 40}, {"L": 40}), ({"L": 100}, {"L": 100})):
        assert plan(*case(**kw), **pk, opts=sr.make_options(MF, 0)) == MF, kw
        for tile in (1, 3, 5, 7):
            assert plan(*case(**kw), **pk, opts=sr.make_options(MF, tile)) == -3, (kw, tile)
            assert plan(*case(**kw), **pk, opts=sr.make_options(AUTO, tile)) == -3, (kw, tile)
        assert tile_of(*case(**kw), **pk, opts=sr.make_options(MF, 0))[1:] == (0, 0)
    assert plan(*case(), kept=list(range(30)), opts=sr.make_options(MF, 2)) == -3            # a short kept list: another capacity
    assert plan(*case(), kept=list(range(66)), opts=sr.make_options(MF, 2)) == MF
    assert plan(*case(), opts=sr.make_options(sr.SR_KERNEL_GENERIC, 3)) == sr.SR_KERNEL_GENERIC   # ignored by the generic kernel
    assert tile_of(*case(), opts=sr.make_options(sr.SR_KERNEL_GENERIC, 0)) == (sr.SR_KERNEL_GENERIC, 0, 0)
    lr, coeff, d, out = case()
    assert sr.load().sr_dict_assemble_tile(lr, coeff, d, 72, 5, 4, 3, out, None, 0, None, None, None) == -1


def test_pre_shuffle_layout_is_checked_on_the_host(lib):
    """coeff as the network holds it before its pixel-shuffle layer: [N][L*s*s][h][w]."""
    PS = sr.SR_COEFF_PRE_SHUFFLE

    def ps_case(L=72, k=5, s=4, C=3, h=8, w=16, cd=sr.SR_F16):
        lr, coeff, d, out = case(L=L, k=k, s=s, C=C, h=h, w=w, cd=cd)
        coeff.c, coeff.h, coeff.w = L * s * s, h, w
        return lr, coeff, d, out
    o = lambda kernel=sr.SR_KERNEL_AUTO, tile=0: sr.make_options(kernel, tile, PS)
    assert plan(*ps_case(), opts=o()) == sr.SR_KERNEL_MFMA
    assert plan(*ps_case(), opts=o(sr.SR_KERNEL_GENERIC)) == sr.SR_KERNEL_GENERIC
    assert plan(*ps_case(), kept=[3, 9, 70], opts=o()) == sr.SR_KERNEL_MFMA
    assert plan(*ps_case(), kept=list(range(30)), opts=o()) == sr.SR_KERNEL_GENERIC      # capacities built: 8 and 72
    assert plan(*ps_case(), kept=list(range(30)), opts=o(sr.SR_KERNEL_MFMA)) == -3
    assert plan(*ps_case(s=3), s=3, opts=o()) == sr.SR_KERNEL_MFMA
    assert plan(*ps_case(w=15, s=3), s=3, opts=o()) == sr.SR_KERNEL_GENERIC              # HR width 45: not whole groups
    for kw, pk in (({"cd": sr.SR_F32}, {}), ({"cd": sr.SR_F8E4M3}, {}), ({"k": 7}, {"k": 7}),
                   ({"C": 1}, {"C": 1}), ({"L": 100}, {"L": 100})):
        assert plan(*ps_case(**kw), **pk, opts=o()) == sr.SR_KERNEL_GENERIC, kw
    # bfloat16: the forms with permuted pixel slots only (LR width a multiple of 4), 65 to 72 atoms
    assert plan(*ps_case(cd=sr.SR_BF16), opts=o()) == sr.SR_KERNEL_MFMA
    assert plan(*ps_case(cd=sr.SR_BF16, s=3), s=3, opts=o()) == sr.SR_KERNEL_MFMA
    assert plan(*ps_case(cd=sr.SR_BF16, w=30), opts=o()) == sr.SR_KERNEL_GENERIC
    assert plan(*ps_case(cd=sr.SR_BF16), kept=[3, 9, 70], opts=o()) == sr.SR_KERNEL_GENERIC
    assert plan(*ps_case(), opts=o(sr.SR_KERNEL_MFMA, 3)) == -3                          # no alternative tiles in this layout
    # the planar shape under the pre-shuffle flag, and the other way round, are shape errors
    assert plan(*case(), opts=o()) == -2
    assert plan(*ps_case()) == -2
    bad = ps_case()
    bad[1].c = 72 * 16 - 1
    assert plan(*bad, opts=o()) == -2
    assert plan(*ps_case(), opts=sr.make_options(0, 0, 4)) == -3                          # unknown layout code
    # pixel-major storage [N][H][W][L]: described like the planar tensor; the matrix-core kernel takes all of 72 fp16
    # atoms of 5x5 on three channels with an HR width of whole 128-pixel units, the generic kernel everything else
    pm = lambda kernel=sr.SR_KERNEL_AUTO, tile=0: sr.make_options(kernel, tile, sr.SR_COEFF_PIXEL_MAJOR)
    assert plan(*case(w=64), opts=pm()) == sr.SR_KERNEL_MFMA
    assert plan(*case(w=64), opts=pm(sr.SR_KERNEL_GENERIC)) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=48), opts=pm()) == sr.SR_KERNEL_GENERIC                            # HR width 192
    assert plan(*case(w=48), opts=pm(sr.SR_KERNEL_MFMA)) == -3
    assert plan(*case(w=64), kept=[3, 9, 70], opts=pm()) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=64), kept=list(range(72)), opts=pm()) == sr.SR_KERNEL_MFMA        # the identity list is no list
    assert plan(*case(w=64), kept=list(range(71, -1, -1)), opts=pm()) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=64), opts=pm(sr.SR_KERNEL_MFMA, 3)) == -3                          # no alternative tiles in this layout
    for kw, pk in (({"cd": sr.SR_F32}, {}), ({"cd": sr.SR_BF16}, {}), ({"k": 7}, {"k": 7}), ({"C": 1}, {"C": 1}), ({"L": 64}, {"L": 64})):
        assert plan(*case(w=64, **kw), **pk, opts=pm()) == sr.SR_KERNEL_GENERIC, kw


def test_blocked_layout_is_checked_on_the_host(lib):
    """SR_COEFF_BLOCKED: units of 128 pixels and groups of 8 atoms or the order does not exist; described like the planar tensor."""
    bl = lambda kernel=sr.SR_KERNEL_AUTO, tile=0: sr.make_options(kernel, tile, sr.SR_COEFF_BLOCKED)
    assert plan(*case(w=64), opts=bl()) == sr.SR_KERNEL_MFMA
    assert plan(*case(w=64), opts=bl(sr.SR_KERNEL_GENERIC)) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=48), opts=bl()) == -3                                             # HR width 192: not whole units
    assert plan(*case(w=64, L=70), L=70, opts=bl()) == -3                                 # not whole groups of 8 atoms
    assert plan(*case(w=64), kept=[3, 9, 70], opts=bl()) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=64), kept=list(range(72)), opts=bl()) == sr.SR_KERNEL_MFMA        # the identity list is no list
    assert plan(*case(w=64), opts=bl(sr.SR_KERNEL_MFMA, 3)) == -3                          # no alternative tiles in this layout
    assert plan(*case(w=64, cd=sr.SR_F8E4M3), opts=bl()) == sr.SR_KERNEL_MFMA              # 8-bit coefficients in the same order
    assert plan(*case(w=64, cd=sr.SR_BF16), opts=bl()) == sr.SR_KERNEL_MFMA
    for kw, pk in (({"cd": sr.SR_F32}, {}), ({"k": 7}, {"k": 7}), ({"C": 1}, {"C": 1}), ({"L": 64}, {"L": 64})):
        assert plan(*case(w=64, **kw), **pk, opts=bl()) == sr.SR_KERNEL_GENERIC, kw
    lg = sr.make_options(0, 0, sr.SR_COEFF_BLOCKED, sr.SR_COEFF_LOGITS)
    assert plan(*case(w=64), opts=lg) == sr.SR_KERNEL_MFMA                                # blocked fp16 logits as well
    assert plan(*case(w=64, cd=sr.SR_BF16), opts=lg) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=64), opts=sr.make_options(0, 0, 4)) == -3                          # unknown layout code


def test_logits_option_is_checked_on_the_host(lib):
    """coeff_kind = SR_COEFF_LOGITS: the softmax needs every atom, so no kept list; f32, f16 or bf16 logits."""
    lg = lambda kernel=sr.SR_KERNEL_AUTO, tile=0, layout=sr.SR_COEFF_PLANAR: sr.make_options(kernel, tile, layout, sr.SR_COEFF_LOGITS)
    assert plan(*case(), opts=lg()) == sr.SR_KERNEL_MFMA
    assert plan(*case(), opts=lg(sr.SR_KERNEL_GENERIC)) == sr.SR_KERNEL_GENERIC
    assert plan(*case(L=65), L=65, opts=lg()) == sr.SR_KERNEL_MFMA
    assert plan(*case(L=49), L=49, opts=lg()) == sr.SR_KERNEL_MFMA                       # the capacity of nine groups of eight
    assert plan(*case(cd=sr.SR_BF16), opts=lg()) == sr.SR_KERNEL_MFMA                    # bfloat16 logits
    for kw, pk in (({"cd": sr.SR_F32}, {}), ({"k": 7}, {"k": 7}), ({"C": 1}, {"C": 1}),
                   ({"L": 48}, {"L": 48}), ({"L": 100}, {"L": 100})):
        assert plan(*case(**kw), **pk, opts=lg()) == sr.SR_KERNEL_GENERIC, kw
        assert plan(*case(**kw), **pk, opts=lg(sr.SR_KERNEL_MFMA)) == -3, kw
    assert plan(*case(), kept=[3, 9, 70], opts=lg()) == -3
    assert plan(*case(), kept=list(range(72)), opts=lg()) == -3                          # not even the identity list
    assert plan(*case(cd=sr.SR_F8E4M3), opts=lg()) == -3
    assert plan(*case(), opts=lg(sr.SR_KERNEL_MFMA, 6)) == -3                            # no alternative tiles in this form
    assert plan(*case(), opts=sr.make_options(0, 0, 0, 2)) == -3                         # unknown kind
    def ps_case(s=4, w=16):
        lr, coeff, d, out = case(s=s, w=w)
        coeff.c, coeff.h, coeff.w = 72 * s * s, 8, w
        return lr, coeff, d, out
    for s in (2, 3, 4):                                                                  # before the pixel-shuffle: LR widths that are multiples of 4
        assert plan(*ps_case(s), s=s, opts=lg(layout=sr.SR_COEFF_PRE_SHUFFLE)) == sr.SR_KERNEL_MFMA
    assert plan(*ps_case(4, 18), opts=lg(layout=sr.SR_COEFF_PRE_SHUFFLE)) == sr.SR_KERNEL_GENERIC
    assert plan(*ps_case(4, 18), opts=lg(sr.SR_KERNEL_MFMA, 0, sr.SR_COEFF_PRE_SHUFFLE)) == -3
    assert plan(*case(w=64), opts=lg(layout=sr.SR_COEFF_PIXEL_MAJOR)) == sr.SR_KERNEL_GENERIC
    assert plan(*case(w=64), opts=lg(sr.SR_KERNEL_MFMA, 0, sr.SR_COEFF_PIXEL_MAJOR)) == -3
    o = sr.make_options(0, 0, 0, sr.SR_COEFF_LOGITS)
    o.reserved[3] = 1
    assert plan(*case(), opts=o) == -3                                                   # reserved fields stay zero


def test_list_form_argument_checks(lib):
    """sr_dict_assemble_list(lr, index, value, dict, L, k, scale, channels, entries, out, stream)"""
    def lcase(L=72, k=5, s=4, C=3, h=8, w=16, T=8, vd=sr.SR_F16, io=sr.SR_F32, idt=sr.SR_U8):
        base = 0x10000000
        return (T_(base, io, 1, C, h, w), T_(base + 0x1000000, idt, 1, T, s * h, s * w),
                T_(base + 0x2000000, vd, 1, T, s * h, s * w), T_(base + 0x8000000, sr.SR_F32, 1, L, k, k),
                T_(base + 0x9000000, io, 1, C, s * h, s * w))
    T_ = T
    f = lib.sr_dict_assemble_list

    def call(ts, L=72, k=5, s=4, C=3, T=8):
        lr, idx, val, d, out = ts
        return f(lr, idx, val, d, L, k, s, C, T, out, None)
    assert call(lcase(idt=sr.SR_F16)) == -3                       # indices must be bytes
    assert call(lcase(vd=sr.SR_BF16)) == -3                       # values: f32 or f16
    assert call(lcase(k=4), k=4) == -3
    assert call(lcase(), T=0) == -3 or call(lcase(), T=0) == -2
    assert call(lcase(T=9)) == -2                                 # entries disagree with the tensors
    assert call(lcase(L=257), L=257) == -3
    ts = lcase()
    ts[2].w = 60
    assert call(ts) == -2
    ts = lcase()
    ts[4].data = ts[1].data                                       # the output on top of the index planes
    assert call(ts) == -4
    ts = lcase()
    ts[2].data = 0x12000001
    assert call(ts) == -7
    assert f(None, *lcase()[1:4], 72, 5, 4, 3, 8, lcase()[4], None) == -1
    ts = lcase()
    for t in ts[:3] + ts[4:]:
        t.n = 0
    assert call(ts) == 0                                          # an empty batch: nothing to do
    lr, idx, val, d, out = lcase()
    assert lib.sr_dict_assemble_list_ex(lr, idx, val, d, 72, 5, 4, 3, 8, out, None, 3) == -3      # no such kernel
    lr, idx, val, d, out = lcase(T=17)
    assert lib.sr_dict_assemble_list_ex(lr, idx, val, d, 72, 5, 4, 3, 17, out, None, sr.SR_KERNEL_MFMA) == -3   # 16 entries at most there
    lr, idx, val, d, out = lcase(vd=sr.SR_F32)
    assert lib.sr_dict_assemble_list_ex(lr, idx, val, d, 72, 5, 4, 3, 8, out, None, sr.SR_KERNEL_MFMA) == -3    # f16 values only


def test_tall_frames_stop_where_the_launch_grids_do(lib):
    def tall(h):
        ts = case(h=h, w=1, C=1)
        for i, t in enumerate(ts):
            t.data = 0x1000000000 * (i + 1)
        return ts
    G = sr.make_options(sr.SR_KERNEL_GENERIC)
    assert plan(*tall(65535), C=1, opts=G) == sr.SR_KERNEL_GENERIC      # 262140 HR rows: the most grid.y holds
    assert plan(*tall(65536), C=1, opts=G) == -3
    assert plan(*tall(65536), C=1) == -3


def test_plan_for_bfloat16_coefficients(lib):
    BF = sr.SR_BF16
    assert plan(*case(cd=BF)) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=BF, C=1), C=1) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=BF, C=2), C=2) == sr.SR_KERNEL_MFMA             # two and four channels: 5x5 only
    assert plan(*case(cd=BF, C=4, k=7), C=4, k=7) == sr.SR_KERNEL_GENERIC
    assert plan(*case(cd=BF, k=3), k=3) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=BF, k=7, L=128), k=7, L=128) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=BF, k=7, L=128, C=1), k=7, L=128, C=1) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=BF, C=5), C=5) == sr.SR_KERNEL_GENERIC
    assert plan(*case(cd=BF, L=73), L=73) == sr.SR_KERNEL_MFMA
    assert plan(*case(cd=BF, L=129), L=129) == sr.SR_KERNEL_GENERIC
    assert plan(*case(cd=BF), kept=[0, 3, 9]) == sr.SR_KERNEL_MFMA
    lr, coeff, d, out = case(cd=BF)
    coeff.data = 0x11000001                                              # two-byte elements need two-byte alignment
    assert plan(lr, coeff, d, out) == -7
    lrb, coeff, d, out = case(io=BF)
    assert plan(lrb, coeff, d, out) == -3                                # images cannot be bfloat16
    lr, coeff, d, out = case()
    assert plan(lr, coeff, T(0x18000000, BF, 1, 72, 5, 5), out) == -3    # nor the dictionary


def test_null_pointers(lib):
    lr, coeff, d, out = case()
    assert plan(None, coeff, d, out) == -1
    assert plan(lr, None, d, out) == -1
    assert plan(lr, coeff, None, out) == -1
    assert plan(lr, coeff, d, None) == -1
    lr.data = None
    assert plan(lr, coeff, d, out) == -1


def test_shape_mismatches(lib):
    assert plan(*case(), L=71) == -2
    assert plan(*case(), C=1) == -2
    assert plan(*case(), s=2) == -2
    lr, coeff, d, out = case()
    out.w += 1
    assert plan(lr, coeff, d, out) == -2
    lr, coeff, d, out = case()
    d.h = 7
    assert plan(lr, coeff, d, out) == -2
    lr, coeff, d, out = case()
    coeff.n = 2
    assert plan(lr, coeff, d, out) == -2


def test_unsupported(lib):
    assert plan(*case(k=4), k=4) == -3       # even k
    assert plan(*case(k=9), k=9) == -3
    assert plan(*case(s=5), s=5) == -3
    assert plan(*case(s=1), s=1) == -3
    assert plan(*case(L=257), L=257) == -3
    assert plan(*case(C=17), C=17) == -3
    lr, coeff, d, out = case()
    out.dtype = sr.SR_F16                      # out dtype must follow lr
    assert plan(lr, coeff, d, out) == -3
    lr, coeff, d, out = case()
    d.dtype = sr.SR_F16
    assert plan(lr, coeff, d, out) == -3
    o = sr.make_options()
    o.reserved[2] = 1
    assert plan(*case(), opts=o) == -3
    assert plan(*case(cd=sr.SR_F8E4M3, k=7, L=16), k=7, L=16, opts=sr.make_options(sr.SR_KERNEL_MFMA)) == -3
    assert plan(*case(C=5), C=5, opts=sr.make_options(sr.SR_KERNEL_MFMA)) == -3


def test_alias_and_alignment(lib):
    lr, coeff, d, out = case()
    out.data = coeff.data + 64
    assert plan(lr, coeff, d, out) == -4
    lr, coeff, d, out = case()
    out.data = lr.data
    assert plan(lr, coeff, d, out) == -4
    lr, coeff, d, out = case()
    coeff.data += 1
    assert plan(lr, coeff, d, out) == -7


def test_kept_lists(lib):
    assert plan(*case(), kept=[0, 5, 71]) > 0
    assert plan(*case(), kept=[0, 72]) == -5
    assert plan(*case(), kept=[-1]) == -5
    assert plan(*case(), kept=[3, 3]) == -5
    assert plan(*case(), kept=list(range(72)) + [0]) == -5
    lr, coeff, d, out = case()
    empty = (ctypes.c_int * 1)(0)
    assert sr.load().sr_dict_assemble_plan(lr, coeff, d, 72, 5, 4, 3, out, empty, 0, None) == -5
    # the selective entry point needs a list
    assert sr.load().sr_dict_assemble_selective(lr, coeff, d, 72, 5, 4, 3, out, None, None, 0, None) == -1


def test_errors_launch_nothing_through_the_real_entry_points(lib):
    """Bad arguments come back as statuses from the launching entry points too
    (they return before any HIP call, so this is safe without a GPU)."""
    lr, coeff, d, out = case()
    assert lib.sr_dict_assemble(lr, coeff, d, 71, 5, 4, 3, out, None) == -2
    assert lib.sr_dict_assemble(None, coeff, d, 72, 5, 4, 3, out, None) == -1
    assert lib.sr_bicubic_upsample(lr, 5, 3, out, None) == -3
    assert lib.sr_bicubic_upsample(lr, 2, 3, out, None) == -2
    assert lib.sr_bicubic_upsample(None, 2, 3, out, None) == -1


def test_empty_batches_are_noops(lib):
    lr, coeff, d, out = case()
    for t in (lr, coeff, out):
        t.n = 0
    assert lib.sr_dict_assemble(lr, coeff, d, 72, 5, 4, 3, out, None) == 0
    assert lib.sr_bicubic_upsample(lr, 4, 3, out, None) == 0


def test_probe_argument_checks_launch_nothing(lib):
    vp = ctypes.c_void_p
    good, sink = vp(0x10000000), vp(0x20000000)
    assert lib.sr_probe_read(None, 1024, sink, None) == -1
    assert lib.sr_probe_read(good, 1024, None, None) == -1
    assert lib.sr_probe_read(good, 1000, sink, None) == -3          # not a multiple of 16 bytes
    assert lib.sr_probe_read(vp(0x10000004), 1024, sink, None) == -7
    assert lib.sr_probe_read(good, 0, sink, None) == 0               # empty: nothing to launch
    assert lib.sr_probe_mix(None, 72, 1280, sink, 3, None) == -1
    assert lib.sr_probe_mix(good, 70, 1280, sink, 3, None) == -3     # plane count not built
    assert lib.sr_probe_mix(good, 72, 1000, sink, 3, None) == -3     # not whole 128-pixel runs
    assert lib.sr_probe_mix(good, 72, 1280, sink, 5, None) == -3
    assert lib.sr_probe_mix(good, 72, 1280, vp(0x20000008), 3, None) == -7
    assert lib.sr_probe_mix(good, 128, 0, sink, 1, None) == 0
    assert lib.sr_probe_mix_tiled(None, 72, 16, 128, 16, sink, 3, None) == -1
    assert lib.sr_probe_mix_tiled(good, 72, 16, 100, 16, sink, 3, None) == -3    # not whole 128-pixel rows
    assert lib.sr_probe_mix_tiled(good, 72, 16, 128, 0, sink, 3, None) == -3     # no such tile
    assert lib.sr_probe_mix_tiled(good, 70, 16, 128, 16, sink, 3, None) == -3
    assert lib.sr_probe_mix_tiled(good, 72, 16, 128, 16, sink, 5, None) == -3
    assert lib.sr_probe_mix_tiled(good, 72, 0, 128, 16, sink, 3, None) == 0
    assert lib.sr_probe_mix_tiled_bytes(good, 72, 4, 16, 128, 16, sink, 3, None) == -3   # one or two bytes per coefficient
    assert lib.sr_probe_mix_tiled_bytes(None, 72, 1, 16, 128, 16, sink, 3, None) == -1
    assert lib.sr_probe_mix_tiled_bytes(good, 72, 1, 0, 128, 16, sink, 3, None) == 0
    assert lib.sr_probe_mix_tiled_paced(good, 72, 2, 16, 128, 16, sink, 3, -1, None) == -3
    assert lib.sr_probe_mix_tiled_paced(good, 72, 2, 0, 128, 16, sink, 3, 16, None) == 0
    # sr_probe_stream(src, read_bytes, dst, write_bytes, blocks, writer_every, lds_bytes, nt_store, sink, stream)
    ps = lib.sr_probe_stream
    assert ps(None, 1024, good, 1024, 26, 13, 0, 0, sink, None) == -1
    assert ps(good, 1024, None, 1024, 26, 13, 0, 0, sink, None) == -1
    assert ps(good, 1024, good, 1024, 26, 13, 0, 0, None, None) == -1
    assert ps(good, 1000, None, 0, 26, 0, 0, 0, sink, None) == -3             # not a multiple of 16 bytes
    assert ps(good, 1024, good, 1024, 26, 0, 0, 0, sink, None) == -3          # bytes to write, nobody to write them
    assert ps(good, 1024, good, 1024, 26, 1, 0, 0, sink, None) == -3          # bytes to read, only writers
    assert ps(good, 1024, good, 1024, 5, 13, 0, 0, sink, None) == -3          # fewer workgroups than one writer needs
    assert ps(good, 1024, None, 0, 0, 0, 0, 0, sink, None) == -3
    assert ps(good, 1024, None, 0, 8, 0, 161 * 1024, 0, sink, None) == -3     # more LDS than a CU has
    assert ps(vp(0x10000008), 1024, None, 0, 8, 0, 0, 0, sink, None) == -7
    assert ps(None, 0, None, 0, 8, 0, 0, 0, sink, None) == 0                  # nothing to do
    # sr_probe_pattern(src, dst, pixels, read_planes, write_planes, same_wave, blocks, writer_every, pad, sink, stream)
    pp = lib.sr_probe_pattern
    assert pp(None, good, 512, 1, 1, 1, 8, 0, 0, sink, None) == -1
    assert pp(good, good, 500, 1, 1, 1, 8, 0, 0, sink, None) == -3            # not whole runs
    assert pp(good, good, 512, 5, 1, 1, 8, 0, 0, sink, None) == -3
    assert pp(good, good, 512, 1, 4, 1, 8, 0, 0, sink, None) == -3
    assert pp(good, good, 512, 2, 1, 0, 26, 13, 0, sink, None) == -3          # 16-byte plane reads: same-wave form only
    assert pp(good, good, 512, 1, 1, 0, 26, 1, 0, sink, None) == -3           # every workgroup a writer
    assert pp(good, good, 512, 0, 1, 1, 8, 0, 128, sink, None) == -3          # padding without plane reads
    assert pp(good, good, 512, 1, 1, 1, 8, 0, 24, sink, None) == -3
    assert pp(good, vp(0x20000004), 512, 1, 1, 1, 8, 0, 0, sink, None) == -7
    assert pp(good, good, 0, 1, 1, 1, 8, 0, 0, sink, None) == 0
    # sr_probe_policy(src, dst, pixels, load_policy, store_policy, flush_every, blocks, sink, stream) and its bit form
    assert lib.sr_probe_policy(good, good, 128, 4, 0, 0, 8, sink, None) == -3
    assert lib.sr_probe_policy(good, good, 128, 0, 0, 0, 7, sink, None) == -3   # one flushing wavefront per XCD needs 8 workgroups
    assert lib.sr_probe_policy(good, None, 128, 0, 0, 0, 8, sink, None) == -1
    assert lib.sr_probe_policy(good, good, 0, 0, 0, 0, 8, sink, None) == 0
    assert lib.sr_probe_policy_bits(good, good, 128, 8, 0, 8, sink, None) == -3
    assert lib.sr_probe_policy_bits(good, good, 100, 0, 0, 8, sink, None) == -3
    assert lib.sr_probe_policy_bits(None, good, 128, 0, 0, 8, sink, None) == -1
    assert lib.sr_probe_policy_bits(good, good, 0, 7, 7, 8, sink, None) == 0


def test_e4m3_coefficients_are_a_coefficient_format_only(lib):
    F8 = sr.SR_F8E4M3
    assert F8 == 2
    lr, coeff, d, out = case(cd=F8)
    assert plan(lr, coeff, d, out) == sr.SR_KERNEL_MFMA              # 5x5, 72 atoms, width % 4 == 0
    lr, coeff, d, out = case(cd=F8, w=15)                             # HR width 60 is fine, 4-byte loads
    assert plan(lr, coeff, d, out) == sr.SR_KERNEL_MFMA
    lr, coeff, d, out = case(cd=F8, s=2, w=15)                        # HR width 30: not whole groups, under 128
    assert plan(lr, coeff, d, out, s=2) == sr.SR_KERNEL_GENERIC
    lr, coeff, d, out = case(cd=F8, s=2, w=75)                        # HR width 150
    assert plan(lr, coeff, d, out, s=2) == sr.SR_KERNEL_MFMA
    lr, coeff, d, out = case(cd=F8, io=sr.SR_F16, C=1, h=3, w=5)      # fp16 image with an odd element count
    assert plan(lr, coeff, d, out, C=1) == sr.SR_KERNEL_GENERIC
    lr, coeff, d, out = case(cd=F8, io=sr.SR_F16, C=1, h=3, w=6)
    assert plan(lr, coeff, d, out, C=1) == sr.SR_KERNEL_MFMA
    lr, coeff, d, out = case(cd=F8, k=7, L=100)
    assert plan(lr, coeff, d, out, L=100, k=7) == sr.SR_KERNEL_MFMA          # 7x7: 17 to 128 atoms
    lr, coeff, d, out = case(cd=F8, k=7, L=200)
    assert plan(lr, coeff, d, out, L=200, k=7) == sr.SR_KERNEL_GENERIC
    coeff_odd = T(0x11000001, F8, 1, 72, 32, 64)                      # one-byte elements: any address
    assert plan(lr, coeff_odd, T(0x18000000, sr.SR_F32, 1, 72, 5, 5), out) == sr.SR_KERNEL_MFMA
    lr8, coeff, d, out = case(io=F8)
    assert plan(lr8, coeff, d, out) == -3                             # images cannot be E4M3
    lr, coeff, d, out = case()
    assert plan(lr, coeff, T(0x18000000, F8, 1, 72, 5, 5), out) == -3  # nor the dictionary


def test_matrix_core_kernel_declines_tensors_beyond_32_bit_offsets(lib):
    def big(L, cd, n=1, h=2048, w=1024):
        lr = T(0x10000000, sr.SR_F32, n, 3, h, w)
        coeff = T(0x1000000000, cd, n, L, 4 * h, 4 * w)
        d = T(0x80000000, sr.SR_F32, 1, L, 5, 5)
        out = T(0x4000000000, sr.SR_F32, n, 3, 4 * h, 4 * w)
        return lr, coeff, d, out
    # 72 planes of 8192 x 4096 fp32 = 9 GiB: plane offsets no longer fit 32 bits
    # (fp16 coefficients, 5x5, three channels have instantiations with element offsets)
    lr, coeff, d, out = big(72, sr.SR_F32)
    assert plan(lr, coeff, d, out) == sr.SR_KERNEL_GENERIC
    assert plan(lr, coeff, d, out, opts=sr.make_options(sr.SR_KERNEL_MFMA, 0)) == -3
    lr, coeff, d, out = big(72, sr.SR_F16)
    assert plan(lr, coeff, d, out) == sr.SR_KERNEL_MFMA
    # the same frame with 40 atoms (2.5 GiB) still qualifies
    lr, coeff, d, out = big(40, sr.SR_F16)
    assert plan(lr, coeff, d, out, L=40) == sr.SR_KERNEL_MFMA
    # ... and as 8-bit coefficients all 72 planes do (2.25 GiB)
    lr, coeff, d, out = big(72, sr.SR_F8E4M3)
    assert plan(lr, coeff, d, out) == sr.SR_KERNEL_MFMA
    # a batch whose fp32 output exceeds 2^32 bytes: image bases are 64-bit, only one image's size counts
    lr, coeff, d, out = big(8, sr.SR_F16, n=44, h=540, w=960)
    assert plan(lr, coeff, d, out, L=8) == sr.SR_KERNEL_MFMA
