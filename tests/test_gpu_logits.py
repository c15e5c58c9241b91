"""Coefficients handed over as LOGITS (sr_options.coeff_kind = SR_COEFF_LOGITS; an extension beyond the paper): the
HIP path applies the per-pixel softmax over the atoms itself, its exponentials rounded to binary16 before the sum
and the fold, and must give what the oracle gives for that reading.

Tolerance.  Both sides round exp(z - max) to binary16; the oracle evaluates it in double, the GPU in fp32 with the
hardware's exponential after one multiply-add (a relative error of a few 1e-7).  A value within that distance of a
rounding boundary, about one in a thousand, rounds the other way: one binary16 step, at most 2^-10 relative, in that
coefficient, which moves the output by Phi_l * 2^-10 * |D_l.B - y|.  So
  * every element: |gpu - ref| <= LOGIT_STEP * max(1, |ref|), LOGIT_STEP = 2.5e-4 (a step in a coefficient of 0.25
    against a response 1 away from the output), plus half an fp16 unit for an fp16 image,
  * nearly all elements are untouched by a step in a large coefficient: at most one in a thousand may exceed the 2e-5
    rule of stored fp16 coefficients (measured on frames of 92 000 pixels: none does, the worst error is 6e-6),
  * and the GPU must be closer to this oracle than to the plain softmax without the rounding (a sharpness check:
    the two differ by 2^-12 relative per coefficient)."""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth
from test_gpu_parity import DEV, GENERIC, MFMA, host, parity_bound

pytestmark = pytest.mark.gpu
LOGITS = sr.SR_COEFF_LOGITS
LOGIT_STEP = 2.5e-4


def run(inp, wl, z, kernel, layout=sr.SR_COEFF_PLANAR, kind=LOGITS):
    out = torch.full((wl.n, wl.c, wl.H, wl.W), float("nan"), device=DEV, dtype=inp["lr"].dtype)
    opts = sr.make_options(kernel, 0, layout, kind)
    if sr.sr_dict_assemble_plan(inp["lr"], z, inp["dict"], wl.L, wl.k, wl.scale, wl.c, out, opts=opts) != kernel:
        return None
    sr.sr_dict_assemble_ex(inp["lr"], z, inp["dict"], wl.L, wl.k, wl.scale, wl.c, out, opts=opts)
    torch.cuda.synchronize()
    return out


def assert_logits_parity(got, ref, out_f16, what):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    half_ulp = 2.0 ** -11 * np.maximum(np.abs(ref), 2.0 ** -14) if out_f16 else 0.0
    worst = float((err / np.maximum(1.0, np.abs(ref))).max(initial=0.0))
    assert (err <= LOGIT_STEP * np.maximum(1.0, np.abs(ref)) + half_ulp).all(), f"{what}: worst error {worst:.3e}"
    beyond = float((err > parity_bound(ref, "f16", out_f16)).mean()) if err.size else 0.0
    assert beyond <= 1e-3, f"{what}: {100 * beyond:.3f} % of the elements are beyond the 2e-5 rule"
    return worst, beyond


CASES = [
    # (N, C, h, w, scale, L, k, logit dtype, image dtype, logit variance)
    (1, 3, 37, 64, 4, 72, 5, "f16", "f32", 1.0),        # the matrix-core family: two tile columns, ragged rows
    (2, 3, 50, 96, 4, 72, 5, "f16", "f32", 2.0),        # two images, three tile columns, wider logits
    (1, 3, 41, 64, 2, 72, 5, "f16", "f32", 1.0),        # scale 2
    (1, 3, 29, 128, 3, 72, 5, "f16", "f16", 1.0),       # scale 3, fp16 image
    (1, 3, 9, 32, 4, 72, 5, "f16", "f32", 1.0),         # fewer rows than a tile
    (1, 3, 20, 33, 4, 72, 5, "f16", "f32", 1.0),        # HR width 132: the last tile column moved left
    (1, 3, 21, 34, 4, 65, 5, "f16", "f32", 1.0),        # 65 planes: seven padding atoms in the last group
    (1, 3, 21, 34, 4, 70, 5, "f16", "f32", 9.0),        # 70 planes; a few atoms dominate
    (1, 3, 21, 36, 3, 50, 5, "f16", "f32", 1.0),        # 50 planes: 22 padding atoms, two whole groups among them
    (1, 3, 37, 64, 4, 72, 5, "bf16", "f32", 1.0),       # bfloat16 logits on the matrix cores
    (2, 3, 29, 128, 3, 72, 5, "bf16", "f16", 4.0),
    (1, 3, 21, 36, 2, 66, 5, "bf16", "f32", 1.0),
    (1, 3, 18, 32, 4, 40, 5, "f16", "f32", 1.0),        # 40 atoms: generic kernel
    (1, 1, 19, 23, 4, 40, 5, "f32", "f32", 1.0),        # fp32 logits
    (2, 2, 16, 21, 3, 17, 7, "bf16", "f16", 1.0),       # bfloat16 logits, 7x7 atoms
    (1, 3, 18, 20, 2, 30, 3, "f16", "f32", 4.0),
    (1, 4, 12, 16, 2, 1, 5, "f16", "f32", 1.0),         # a single atom: its coefficient is one whatever the logit
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%dC%dh%dw%ds%dL%dk%d%s%s-v%g" % c)
def test_logits_against_the_oracle(oracle, case):
    N, C, h, w, s, L, k, cd, io, var = case
    wl = sr_synth.Workload("lg", 53, N, C, h, w, s, L, k, cd, io, 0.0, var)
    inp = sr_synth.make_inputs(wl, DEV)
    z = sr_synth.make_logits(wl, DEV)
    hi = host(inp)
    zh = sr_synth.stored_numpy(z)
    ref = oracle.dict_assemble(hi["lr"], zh, hi["dict"], s, logits=True)
    plain = oracle.assemble(oracle.bicubic(hi["lr"], s), oracle.softmax_logits(zh, round_half=False), hi["dict"])
    ran = 0
    for kernel in (GENERIC, MFMA):
        got = run(inp, wl, z, kernel)
        if got is None:
            continue
        ran += 1
        assert not torch.isnan(got).any(), "some output pixel was never written"
        g = got.float().cpu().numpy()
        assert_logits_parity(g, ref, io == "f16", f"kernel {kernel}")
        if L > 1 and io == "f32":
            rms_ref, rms_plain = np.sqrt(np.mean((g - ref) ** 2)), np.sqrt(np.mean((g - plain) ** 2))
            assert rms_ref < 0.5 * rms_plain, f"kernel {kernel}: as close to the unrounded softmax ({rms_plain:.2e}) as to the rounded one ({rms_ref:.2e})"
    assert ran >= 1
    takes = run(inp, wl, z, MFMA) is not None
    assert takes == (cd in ("f16", "bf16") and C == 3 and k == 5 and 49 <= L <= 72)


@pytest.mark.parametrize("cd", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(1, 23, 64, 4, 72), (2, 19, 96, 3, 72), (1, 21, 64, 2, 72), (1, 9, 36, 3, 65), (1, 30, 68, 4, 50)],
                         ids=lambda c: "N%dh%dw%ds%dL%d" % c)
def test_logits_before_the_pixel_shuffle_on_the_matrix_cores(oracle, shape, cd):
    """What the network's last convolution writes when the normalisation is left to the call: logits in the layout
    before the pixel-shuffle.  Against the oracle (shuffle, then softmax, then the definition) and, bit for bit,
    against the call with the shuffled logits."""
    N, h, w, s, L = shape
    wl = sr_synth.Workload("lg", 57, N, 3, h, w, s, L, 5, cd, "f32", 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    z = sr_synth.make_logits(wl, DEV)
    pre = sr_synth.to_pre_shuffle(z, s)
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(pre), hi["dict"], s, logits=True, pre_shuffle=True)
    got = run(inp, wl, pre, MFMA, sr.SR_COEFF_PRE_SHUFFLE)
    assert got is not None and not torch.isnan(got).any()
    assert_logits_parity(got.cpu().numpy(), ref, False, "pre-shuffle logits")
    assert torch.equal(got, run(inp, wl, z, MFMA))


@pytest.mark.parametrize("shape", [(1, 23, 64, 4), (2, 19, 128, 3), (1, 21, 64, 2), (1, 5, 32, 4)], ids=lambda c: "N%dh%dw%ds%d" % c)
def test_logits_in_the_blocked_order_on_the_matrix_cores(oracle, shape):
    """Logits stored in the blocked order (the matrix-core kernel's own operand order): against the oracle (blocked to planar,
    softmax, the definition) and, bit for bit, against the call with the planar logits."""
    N, h, w, s = shape
    wl = sr_synth.Workload("lg", 59, N, 3, h, w, s, 72, 5, "f16", "f32", 0.0, 2.0)
    inp = sr_synth.make_inputs(wl, DEV)
    z = sr_synth.make_logits(wl, DEV)
    blk = sr_synth.to_blocked(z)
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(blk), hi["dict"], s, logits=True, blocked=True)
    got = run(inp, wl, blk, MFMA, sr.SR_COEFF_BLOCKED)
    assert got is not None and not torch.isnan(got).any()
    assert_logits_parity(got.cpu().numpy(), ref, False, "blocked logits")
    assert torch.equal(got, run(inp, wl, z, MFMA))
    gen = run(inp, wl, blk, GENERIC, sr.SR_COEFF_BLOCKED)
    assert_logits_parity(gen.cpu().numpy(), ref, False, "blocked logits, generic kernel")
    # the shift is the pixel's own largest logit (any other shift rounds the exponentials elsewhere): as close to the oracle
    # as the planar call of the same kernel, and closer to it than to the softmax without the rounding
    plain = oracle.assemble(oracle.bicubic(hi["lr"], s), oracle.softmax_logits(sr_synth.stored_numpy(z), round_half=False), hi["dict"])
    for name, t in (("matrix-core", got), ("generic", gen)):
        g = t.cpu().numpy().astype(np.float64)
        rms_ref, rms_plain = np.sqrt(np.mean((g - ref) ** 2)), np.sqrt(np.mean((g - plain) ** 2))
        assert rms_ref < 0.5 * rms_plain, f"{name}: rms {rms_ref:.2e} against the rounded form, {rms_plain:.2e} against the unrounded one"
    assert torch.equal(gen, run(inp, wl, z, GENERIC))


def test_logits_in_the_other_layouts_run_on_the_generic_kernel(oracle):
    wl = sr_synth.Workload("lg", 54, 1, 3, 12, 30, 4, 72, 5, "f16", "f32", 0.0, 1.0)   # LR width not a multiple of 4
    inp = sr_synth.make_inputs(wl, DEV)
    z = sr_synth.make_logits(wl, DEV)
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(z), hi["dict"], wl.scale, logits=True)
    for layout, moved, flag in ((sr.SR_COEFF_PRE_SHUFFLE, sr_synth.to_pre_shuffle(z, wl.scale), "pre_shuffle"),
                                (sr.SR_COEFF_PIXEL_MAJOR, sr_synth.to_pixel_major(z), "pixel_major")):
        assert run(inp, wl, moved, MFMA, layout) is None
        got = run(inp, wl, moved, GENERIC, layout)
        assert_logits_parity(got.cpu().numpy(), ref, False, flag)
        assert np.sqrt(np.mean((got.cpu().numpy() - ref) ** 2)) < 2e-7, flag      # (a wrong shift would leave 1e-6)
        again = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(moved), hi["dict"], wl.scale, logits=True, **{flag: True})
        assert np.array_equal(again, ref)
        assert torch.equal(got, run(inp, wl, z, GENERIC))


@pytest.mark.parametrize("cd", ["f16", "bf16"])
def test_masked_atoms_and_shifted_logits(oracle, cd):
    """Logits of minus infinity are atoms switched off (coefficient zero); a common shift of a pixel's logits changes
    nothing; logits far from zero do not overflow."""
    wl = sr_synth.Workload("lg", 55, 1, 3, 16, 32, 4, 72, 5, cd, "f32", 0.0, 1.0)
    inp = sr_synth.make_inputs(wl, DEV)
    z = sr_synth.make_logits(wl, DEV)
    g = torch.Generator(device="cpu").manual_seed(7)
    mask = (torch.rand(z.shape, generator=g) < 0.3).to(DEV)
    mask[:, 5] = False                                   # every pixel keeps an atom
    mask[:, 0, :8] = True                                # the first plane a lane half loads starts some maxima switched off
    mask[:, 1, 4:12] = True
    zm = z.masked_fill(mask, float("-inf"))
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(zm), hi["dict"], wl.scale, logits=True)
    for kernel in (GENERIC, MFMA):
        got = run(inp, wl, zm, kernel)
        assert got is not None and torch.isfinite(got).all()
        assert_logits_parity(got.cpu().numpy(), ref, False, f"masked, kernel {kernel}")
    # multiples of 1/8 keep the shifted logits exact in fp16
    # (bfloat16: multiples of 1/8 up to 16)
    zq = (torch.round(z.float() * 8.0) / 8.0).to(z.dtype)
    span = 200 if cd == "f16" else 8
    shift = torch.randint(-span, span, (1, 1, wl.H, wl.W), generator=g).to(DEV).to(z.dtype)
    for kernel in (GENERIC, MFMA):
        a, b = run(inp, wl, zq, kernel), run(inp, wl, zq + shift, kernel)
        # (the shift enters the exponent as -max * log2(e), rounded once: a few units in the last place of fp32)
        assert torch.isfinite(b).all() and (a - b).abs().max().item() <= LOGIT_STEP


def test_random_shapes_the_two_kernels_agree_on_logits():
    """Seeded random frames, scales, atom counts 49 to 72, both 16-bit types, both layouts: the matrix-core form against
    the generic kernel.  Both evaluate the same fp32 expression for an exponential, so they round it the same way and
    differ by fp32 summation order only."""
    rng = np.random.default_rng(77)
    compared = 0
    for index in range(120):
        s = int(rng.choice([2, 3, 4]))
        h, w = int(rng.integers(1, 60)), int(rng.integers(1, 100))
        L, N = int(rng.integers(49, 73)), int(rng.choice([1, 1, 2, 3]))
        cd, io = str(rng.choice(["f16", "bf16"])), str(rng.choice(["f32", "f16"]))
        wl = sr_synth.Workload("lgr", 300 + index, N, 3, h, w, s, L, 5, cd, io, 0.0, float(rng.choice([0.5, 1.0, 4.0])))
        inp = sr_synth.make_inputs(wl, DEV)
        z = sr_synth.make_logits(wl, DEV)
        layout = sr.SR_COEFF_PLANAR
        if rng.random() < 0.4:
            z, layout = sr_synth.to_pre_shuffle(z, s), sr.SR_COEFF_PRE_SHUFFLE
        a = run(inp, wl, z, MFMA, layout)
        if a is None:
            continue                                    # narrow ragged frames, LR widths the permuted forms do not take
        b = run(inp, wl, z, GENERIC, layout)
        assert torch.isfinite(a).all(), f"{wl}: some output pixel was never written"
        tol = (5e-5 + (2.0 ** -10 if io == "f16" else 0.0)) * max(1.0, float(b.abs().max()))
        err = float((a.float() - b.float()).abs().max())
        assert err <= tol, f"{wl} layout {layout}: kernels differ by {err:.3e} > {tol:.1e}"
        compared += 1
    assert compared >= 40, compared


def test_random_small_shapes_against_the_oracle(oracle):
    """Seeded random small cases over everything the call takes with logits (kernel sizes, channel counts, atom counts from
    one up, the three logit types, the three layouts, batches, ragged sizes): every kernel that takes the case against the
    oracle."""
    rng = np.random.default_rng(78)
    ran = {GENERIC: 0, MFMA: 0}
    for index in range(48):
        k, s = int(rng.choice([3, 5, 5, 7])), int(rng.choice([2, 3, 4]))
        C, N = int(rng.choice([1, 2, 3, 3, 4])), int(rng.choice([1, 1, 2, 3]))
        L = int(rng.integers(1, 73)) if rng.random() < 0.6 else int(rng.integers(49, 73))
        if k == 5 and C == 3 and rng.random() < 0.5:
            L = int(rng.integers(49, 73))
        h, w = int(rng.integers(1, 24)), int(rng.integers(1, 40))
        cd, io = str(rng.choice(["f16", "f16", "bf16", "f32"])), str(rng.choice(["f32", "f16"]))
        wl = sr_synth.Workload("lgs", 500 + index, N, C, h, w, s, L, k, cd, io, 0.0, float(rng.choice([1.0, 3.0])))
        inp = sr_synth.make_inputs(wl, DEV)
        z = sr_synth.make_logits(wl, DEV)
        hi = host(inp)
        ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(z), hi["dict"], s, logits=True)
        layout, moved = sr.SR_COEFF_PLANAR, z
        pick = rng.random()
        if pick < 0.3:
            layout, moved = sr.SR_COEFF_PRE_SHUFFLE, sr_synth.to_pre_shuffle(z, s)
        elif pick < 0.5:
            layout, moved = sr.SR_COEFF_PIXEL_MAJOR, sr_synth.to_pixel_major(z)
        for kernel in (GENERIC, MFMA):
            got = run(inp, wl, moved, kernel, layout)
            if got is None:
                continue
            assert not torch.isnan(got).any(), f"{wl} layout {layout} kernel {kernel}: some output pixel was never written"
            assert_logits_parity(got.float().cpu().numpy(), ref, io == "f16", f"{wl} layout {layout} kernel {kernel}")
            ran[kernel] += 1
    assert ran[GENERIC] == 48 and ran[MFMA] >= 1, ran            # (the matrix-core form has its own random test above)


def test_4k_frame_of_logits(oracle):
    """The headline frame handed over as logits, in the launch configuration the benchmark times: sampled pixels
    (corners and edges among them) against the oracle, and the whole frame against the frame computed from the
    coefficients the generator derives from the same logits (its softmax stored as fp16: another rounding, so only
    to fp16's relative precision)."""
    wl = sr_synth.WORKLOADS["4k_dense"]
    inp = sr_synth.make_inputs(wl, DEV)
    from test_gpu_parity import run_gpu
    dense = run_gpu(inp, wl, MFMA)
    del inp["coeff"]
    z = sr_synth.make_logits(wl, DEV)
    got = run(inp, wl, z, MFMA)
    assert got is not None and torch.isfinite(got).all()
    assert (got - dense).abs().max().item() < 1e-3
    # the same logits in the layout before the network's pixel-shuffle: the same bits
    pre = sr_synth.to_pre_shuffle(z, wl.scale)
    assert torch.equal(run(inp, wl, pre, MFMA, sr.SR_COEFF_PRE_SHUFFLE), got)
    del pre
    rng = np.random.default_rng(14)
    npts = 3000
    pts = np.stack([np.zeros(npts, dtype=np.int64), rng.integers(0, wl.H, npts), rng.integers(0, wl.W, npts)], axis=1)
    pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
    pts[4:304, 1] = wl.H - 1 - (pts[4:304, 1] % 25)
    pts[304:604, 2] = wl.W - 1 - (pts[304:604, 2] % 5)
    ys, xs = torch.from_numpy(pts[:, 1]).to(DEV), torch.from_numpy(pts[:, 2]).to(DEV)
    zs = z[0][:, ys, xs].cpu().numpy().reshape(1, wl.L, 1, npts)            # the sampled pixels' logits
    phi_s = oracle.softmax_logits(zs)
    phi = np.zeros((1, wl.L, wl.H, wl.W), dtype=np.float64)                # only the sampled pixels are read
    phi[0][:, pts[:, 1], pts[:, 2]] = phi_s[0, :, 0, :]
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    want = oracle.assemble_points(U, phi, inp["dict"].cpu().numpy(), pts)
    have = got.cpu().numpy()[0][:, pts[:, 1], pts[:, 2]].T
    assert_logits_parity(have, want, False, "sampled pixels")
