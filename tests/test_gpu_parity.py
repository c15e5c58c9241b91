"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same
stored input bytes, element by element.

Tolerances - ONE rule, parity_bound() below, used by every comparison in the GPU tests:
  * fp32 coefficients:  |gpu - ref| <= 1e-5 * max(1, |ref|)                  (the stated target)
  * fp16 / E4M3 coefficients: the stated target is 2e-3 absolute.  Both sides read the SAME
    stored coefficients, widened exactly, so the kernel's own error is only fp32 accumulation
    plus the 2^-22 residue of the two-operand dictionary split: asserted as
    |gpu - ref| <= 2e-5 * max(1, |ref|), a hundred times inside the target - tight enough to
    notice a dictionary rounded to fp16 (5e-4 relative) or a dropped low operand.
  * bfloat16 coefficients: the dictionary enters the matrix cores as two bfloat16 operands, 16
    significant bits, a 2^-17 relative residue per entry: 1e-4 * max(1, |ref|).
  * an fp16 OUTPUT tensor adds its own rounding, half an fp16 ulp of the result:
    + 2^-11 * max(|ref|, 2^-14), whatever the coefficient type.
  Every bound is also checked to lie inside the stated target (2e-3 for 16- and 8-bit
  coefficients with results of order one).
"""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
GENERIC, MFMA = sr.SR_KERNEL_GENERIC, sr.SR_KERNEL_MFMA


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sr.load()


KERNEL_ERROR = {"f32": 1e-5, "f16": 2e-5, "f8": 2e-5, "bf16": 1e-4}
STATED_TARGET_16BIT = 2e-3


def parity_bound(ref, coeff_dtype, out_f16=False):
    """Largest |gpu - ref| accepted per element (the module docstring derives it)."""
    ref = np.abs(np.asarray(ref, dtype=np.float64))
    bound = KERNEL_ERROR[coeff_dtype] * np.maximum(1.0, ref)
    if out_f16:
        bound = bound + 2.0 ** -11 * np.maximum(ref, 2.0 ** -14)
    return bound


def tolerance_ok(got, ref, coeff_dtype, out_f16=False):
    """(worst error relative to max(1, |ref|), the rule's relative part, every element inside its bound)"""
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    ok = bool((err <= parity_bound(ref, coeff_dtype, out_f16)).all())
    if coeff_dtype != "f32" and np.abs(ref).max(initial=0.0) < 4.0:
        ok = ok and bool((err <= STATED_TARGET_16BIT + (2.0 ** -11 * np.abs(ref) if out_f16 else 0.0)).all())
    return float((err / np.maximum(1.0, np.abs(ref))).max(initial=0.0)), KERNEL_ERROR[coeff_dtype], ok


def assert_parity(got, ref, coeff_dtype, out_f16=False, what=""):
    worst, tol, ok = tolerance_ok(got, ref, coeff_dtype, out_f16)
    assert ok, f"{what}: worst error {worst:.3e} (relative to max(1, |ref|)) exceeds the {coeff_dtype} bound {tol:.0e}"
    return worst


def run_gpu(inp, wl, kernel, kept=None, gamma=None, tile=0):
    out = torch.full((wl.n, wl.c, wl.H, wl.W), float("nan"), device=DEV, dtype=inp["lr"].dtype)
    opts = sr.make_options(kernel, tile)
    sr.sr_dict_assemble_ex(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, out,
                           kept=kept, gamma=gamma, opts=opts)
    torch.cuda.synchronize()
    return out


def host(inp):
    return {k: (sr_synth.stored_numpy(v) if torch.is_tensor(v) else v) for k, v in inp.items()}


def planned(inp, wl, kernel, kept=None, tile=0):
    out = torch.empty((wl.n, wl.c, wl.H, wl.W), device=DEV, dtype=inp["lr"].dtype)
    return sr.sr_dict_assemble_plan(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c,
                                    out, kept=kept, opts=sr.make_options(kernel, tile))


def check_full(oracle, wl, kernel, kept=None, gamma=None, inp=None, tile=0):
    inp = inp or sr_synth.make_inputs(wl, DEV)
    if planned(inp, wl, kernel, kept, tile) != kernel:
        pytest.skip("this kernel does not take this case")
    got = run_gpu(inp, wl, kernel, kept, gamma, tile).float().cpu().numpy()
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale, kept=kept, gamma=gamma)
    assert not np.isnan(got).any(), "some output pixel was never written"
    return assert_parity(got, ref, wl.coeff_dtype, wl.lr_dtype == "f16", wl.name)


KERNELS = [pytest.param(GENERIC, id="generic"), pytest.param(MFMA, id="mfma")]


# ---- the stated workloads, whole frames --------------------------------------
@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("name", ["tiny", "720p", "1080p_fp16"])
def test_workload_full_frame(oracle, name, kernel):
    check_full(oracle, sr_synth.WORKLOADS[name], kernel)


@pytest.mark.parametrize("kernel", KERNELS)
def test_video_workload_two_frames(oracle, kernel):
    """L=128, 7x7 atoms, fp16 LR and output; two of the sixteen frames in full."""
    check_full(oracle, sr_synth.scaled(sr_synth.WORKLOADS["video"], n=2), kernel)


def test_video_workload_all_sixteen_frames(oracle):
    """The whole video-stress batch (16 frames, 8.5 GB of coefficients) in one call:
    frame 11 in full and 4000 sampled pixels of the other frames, oracle pixel by
    pixel."""
    wl = sr_synth.WORKLOADS["video"]
    inp = sr_synth.make_inputs(wl, DEV)
    assert planned(inp, wl, sr.SR_KERNEL_AUTO) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO).float().cpu().numpy()
    assert not np.isnan(got).any()
    lr, D = inp["lr"].cpu().numpy(), inp["dict"].cpu().numpy()
    U = oracle.bicubic(lr, wl.scale)
    f = 11
    cf = inp["coeff"][f:f + 1].cpu().numpy()
    ref = oracle.assemble(U[f:f + 1], cf, D)
    assert_parity(got[f:f + 1], ref, "f16", True, "frame 11")
    rng = np.random.default_rng(5)
    for frame in (0, 3, 7, 15):
        pts = np.stack([np.zeros(1000, dtype=np.int64), rng.integers(0, wl.H, 1000), rng.integers(0, wl.W, 1000)], axis=1)
        pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
        cf = inp["coeff"][frame:frame + 1].cpu().numpy()
        want = oracle.assemble_points(U[frame:frame + 1], cf, D, pts)
        have = got[frame][:, pts[:, 1], pts[:, 2]].T
        assert_parity(have, want, "f16", True, f"frame {frame}")


def test_4k_dense_full_frame_in_the_benchmarked_configuration(oracle):
    """The headline workload at full size, default kernel choice (what bench.py
    times), every one of the 3 x 2160 x 3840 outputs against the oracle."""
    wl = sr_synth.WORKLOADS["4k_dense"]
    inp = sr_synth.make_inputs(wl, DEV)
    assert planned(inp, wl, sr.SR_KERNEL_AUTO) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO).cpu().numpy()
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale)
    assert not np.isnan(got).any()
    assert_parity(got, ref, "f16", False, "4k_dense")


def test_4k_dense_fp8_full_frame(oracle):
    """The 4K frame with the coefficients stored as 8-bit E4M3 floats: every output
    against the oracle, which widens the same stored bytes."""
    wl = sr_synth.WORKLOADS["4k_dense_fp8"]
    inp = sr_synth.make_inputs(wl, DEV)
    assert planned(inp, wl, sr.SR_KERNEL_AUTO) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO).cpu().numpy()
    hi = host(inp)
    assert hi["coeff"].dtype == np.uint8
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale)
    assert not np.isnan(got).any()
    assert_parity(got, ref, "f8", False, "4k_dense_fp8")


def test_8k_frame_with_more_than_4_gb_of_coefficients(oracle):
    """1080p x4 -> 7680 x 4320 with 72 fp16 planes: 4.8 GB of coefficients, beyond 32-bit
    byte offsets.  The matrix-core kernel takes it with element offsets: every output of the
    dense call against the oracle, and sampled pixels (corners, last rows and columns
    among them) for kept lists that use the two smaller capacities."""
    wl = sr_synth.WORKLOADS["8k_dense"]
    inp = sr_synth.make_inputs(wl, DEV)
    assert planned(inp, wl, sr.SR_KERNEL_AUTO) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO).cpu().numpy()
    assert not np.isnan(got).any()
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale)
    assert_parity(got, ref, "f16", False, "8k_dense")
    del got, ref
    U = oracle.bicubic(hi["lr"], wl.scale)
    rng = np.random.default_rng(8)
    pts = np.stack([np.zeros(4000, dtype=np.int64), rng.integers(0, wl.H, 4000), rng.integers(0, wl.W, 4000)], axis=1)
    pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
    pts[4:1004, 1] = wl.H - 1 - (pts[4:1004, 1] % 30)            # the last tile rows
    for n_keep in (8, 30):
        kept = sorted(int(v) for v in rng.choice(wl.L, n_keep, replace=False))
        if 71 not in kept:
            kept[-1] = 71                                          # the plane farthest from the base
        gamma = [float(v) for v in rng.uniform(0.5, 1.5, n_keep)]
        assert planned(inp, wl, sr.SR_KERNEL_AUTO, kept) == MFMA
        have = run_gpu(inp, wl, sr.SR_KERNEL_AUTO, kept=kept, gamma=gamma).cpu().numpy()
        want = oracle.assemble_points(U, hi["coeff"], hi["dict"], pts, kept=kept, gamma=gamma)
        assert_parity(have[0][:, pts[:, 1], pts[:, 2]].T, want, "f16", False, f"{n_keep} kept atoms")
    # the same frame with its coefficients as bfloat16: sampled pixels of the dense call
    del inp["coeff"]
    wlb = sr_synth.scaled(wl, coeff_dtype="bf16")
    inp["coeff"] = sr_synth.make_coeff(wlb, DEV)
    assert planned(inp, wlb, sr.SR_KERNEL_AUTO) == MFMA
    have = run_gpu(inp, wlb, sr.SR_KERNEL_AUTO).cpu().numpy()
    assert not np.isnan(have).any()
    want = oracle.assemble_points(U, sr_synth.stored_numpy(inp["coeff"]), hi["dict"], pts)
    assert_parity(have[0][:, pts[:, 1], pts[:, 2]].T, want, "bf16", False, "bfloat16")


def test_4k_dense_bf16_full_frame(oracle):
    """The 4K frame with bfloat16 coefficients: every output against the oracle, which widens
    the same stored bits."""
    wl = sr_synth.WORKLOADS["4k_dense_bf16"]
    inp = sr_synth.make_inputs(wl, DEV)
    assert planned(inp, wl, sr.SR_KERNEL_AUTO) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO).cpu().numpy()
    hi = host(inp)
    assert hi["coeff"].dtype == np.uint16
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale)
    assert not np.isnan(got).any()
    assert_parity(got, ref, "bf16", False, "4k_dense_bf16")


def test_bfloat16_coefficients_beyond_the_fp16_range(oracle):
    """Coefficients of 1e6 and 1e-30 (neither representable in fp16) with atoms scaled to
    bring the result back to order one: both kernels widen bfloat16 exactly."""
    wl = sr_synth.Workload("bfr", 61, 1, 3, 40, 64, 4, 16, 5, "bf16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    scale = torch.tensor([1e6, 1e-30] * 8, device=DEV).view(1, 16, 1, 1)
    inp["coeff"] = (inp["coeff"].float() * scale).to(torch.bfloat16)
    inp["dict"] = inp["dict"] / scale.view(16, 1, 1)
    for kernel in (GENERIC, MFMA):
        assert planned(inp, wl, kernel) == kernel
        got = run_gpu(inp, wl, kernel).cpu().numpy()
        hi = host(inp)
        ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale)
        assert_parity(got, ref, "bf16", False, f"kernel {kernel}")


@pytest.mark.parametrize("cd,io", [("f16", "f32"), ("f8", "f16")])
def test_batch_whose_output_exceeds_32_bit_offsets(oracle, cd, io):
    """Forty-four 4K frames (fp16 images: ninety) with two atoms: the output is 4.4 GB, past
    32-bit byte offsets, while each image is not.  Sampled pixels of the first, the last and
    the image that straddles the 4 GB mark, oracle pixel by pixel."""
    n = 44 if io == "f32" else 90
    wl = sr_synth.Workload("batch", 71, n, 3, 540, 960, 4, 2, 5, cd, io, 0.0, 1.0)
    inp = sr_synth.make_inputs(wl, DEV)
    assert planned(inp, wl, sr.SR_KERNEL_AUTO) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO)
    assert not torch.isnan(got).any()
    lr, D = inp["lr"].float().cpu().numpy(), inp["dict"].cpu().numpy()
    rng = np.random.default_rng(9)
    esz = 4 if io == "f32" else 2
    straddle = (1 << 32) // (3 * wl.H * wl.W * esz)
    assert 0 < straddle < n
    for frame in sorted({0, straddle - 1, straddle, n - 1}):
        U = oracle.bicubic(sr_synth.stored_numpy(inp["lr"][frame:frame + 1]), wl.scale)
        pts = np.stack([np.zeros(800, dtype=np.int64), rng.integers(0, wl.H, 800), rng.integers(0, wl.W, 800)], axis=1)
        pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
        want = oracle.assemble_points(U, sr_synth.stored_numpy(inp["coeff"][frame:frame + 1]), D, pts)
        have = got[frame].float().cpu().numpy()[:, pts[:, 1], pts[:, 2]].T
        assert_parity(have, want, cd, io == "f16", f"frame {frame}")


def test_every_fp8_code_is_widened_as_the_oracle_does(oracle):
    """All 254 finite E4M3 codes, one per pixel, through a single centred delta atom on a
    constant image: the output IS the widened coefficient (both kernels, bit for bit)."""
    codes = [b for b in range(256) if b & 0x7F != 0x7F]
    H, W = 8, 32                                    # 256 HR pixels >= 254 codes
    bits = torch.tensor((codes + [0, 0])[:H * W], dtype=torch.uint8).reshape(1, 1, H, W)
    coeff = bits.view(torch.float8_e4m3fn).to(DEV)
    lr = torch.ones((1, 1, H // 2, W // 2), device=DEV)
    D = torch.zeros((1, 1, 5, 5), device=DEV)
    D[0, 0, 2, 2] = 1.0
    want = np.array([oracle.e4m3_to_double(int(b)) for b in bits.flatten()]).reshape(H, W)
    for kernel in (sr.SR_KERNEL_GENERIC, sr.SR_KERNEL_MFMA):
        out = torch.full((1, 1, H, W), float("nan"), device=DEV)
        sr.sr_dict_assemble_ex(lr, coeff, D, 1, 5, 2, 1, out, opts=sr.make_options(kernel, 0))
        torch.cuda.synchronize()
        assert np.array_equal(out[0, 0].cpu().numpy().astype(np.float64), want), f"kernel {kernel}"


def test_4k_selective_full_frame(oracle):
    """4K with the 8 kept atoms of the selective workload (global kept list)."""
    wl = sr_synth.WORKLOADS["4k_selective"]
    inp = sr_synth.make_inputs(wl, DEV)
    kept = inp["kept"]
    assert planned(inp, wl, sr.SR_KERNEL_AUTO, kept) == MFMA
    got = run_gpu(inp, wl, sr.SR_KERNEL_AUTO, kept=kept).cpu().numpy()
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale, kept=kept)
    assert_parity(got, ref, "f16", False, "4k_selective")
    # about 13 % of the coefficient mass is dropped: the result must differ from dense
    dense = oracle.assemble(oracle.bicubic(hi["lr"], wl.scale), hi["coeff"], hi["dict"], rows=(0, 8))
    assert np.abs(dense[:, :, :8] - ref[:, :, :8]).max() > 1e-2


@pytest.mark.parametrize("tile", range(10))
@pytest.mark.parametrize("shape", [(50, 72, 4), (37, 40, 3), (61, 100, 2)])
def test_every_tile_shape_of_the_matrix_core_kernel(oracle, tile, shape):
    """All built tile shapes (a tuning option) on images that leave ragged tails
    in both directions and span several tiles."""
    h, w, s = shape
    wl = sr_synth.Workload("tiles", 16, 2, 3, h, w, s, 72, 5, "f16", "f32")
    check_full(oracle, wl, MFMA, tile=tile)


# ---- shapes that span several tiles and leave ragged tails --------------------
RAGGED = [
    # (h, w, scale, C, L, k, coeff dtype, io dtype, N)
    (5, 7, 3, 3, 72, 5, "f32", "f32", 1),
    (37, 50, 2, 1, 72, 5, "f16", "f32", 2),
    (33, 26, 4, 3, 72, 5, "f16", "f32", 1),
    (21, 40, 3, 3, 72, 5, "f16", "f32", 1),
    (19, 30, 4, 3, 128, 7, "f16", "f16", 3),
    (11, 13, 2, 2, 5, 3, "f32", "f16", 1),
    (9, 10, 4, 4, 256, 7, "f16", "f32", 1),
    (1, 1, 2, 1, 1, 3, "f32", "f32", 1),
    (1, 2, 4, 3, 72, 5, "f16", "f32", 1),
    (2, 1, 3, 1, 17, 7, "f32", "f32", 1),
    (70, 66, 4, 1, 72, 5, "f16", "f32", 1),
    (45, 64, 4, 3, 40, 5, "f16", "f32", 1),
    (16, 96, 4, 3, 8, 5, "f16", "f32", 1),
    (16, 48, 4, 3, 13, 7, "f16", "f16", 1),
    (23, 27, 4, 3, 72, 5, "f16", "f32", 1),     # HR width 108: multiple of 4, not of 8
    (19, 31, 2, 3, 72, 5, "f16", "f32", 1),     # HR width 62: not whole groups of four and under 128: generic kernel only
    (19, 31, 2, 3, 100, 7, "f16", "f16", 2),    # HR width 62: fine for 7x7 (2 pixels per lane)
    (14, 29, 4, 1, 30, 5, "f16", "f16", 1),     # HR width 116, one channel, fp16 output
    (25, 33, 2, 3, 72, 5, "f32", "f32", 2),     # fp32 coefficients on the fp32 matrix-core path, HR width 66
    (20, 27, 3, 1, 41, 5, "f32", "f16", 1),     # ... HR width 81: odd and under 128: generic kernel only
    (18, 26, 3, 1, 41, 5, "f32", "f16", 1),     # ... HR width 78, one channel, fp16 image
    (31, 45, 4, 3, 9, 5, "f32", "f32", 1),      # ... few atoms
    (6, 8, 2, 16, 9, 3, "f16", "f32", 1),       # the largest channel count accepted
    (60, 128, 4, 3, 24, 5, "f16", "f32", 9),    # 540 tiles over 9 images: every XCD share crosses image borders
    (33, 47, 4, 3, 128, 3, "f16", "f32", 1),    # 128 atoms of 3x3
    (30, 36, 3, 1, 100, 3, "bf16", "f16", 1),   # ... bfloat16, one channel, x3, fp16 image
    (33, 47, 2, 3, 128, 3, "f32", "f32", 1),    # ... fp32 coefficients, x2
    (33, 48, 4, 3, 90, 3, "f8", "f32", 2),      # ... 8-bit coefficients
    (33, 47, 4, 3, 128, 5, "f32", "f32", 2),    # 128 atoms of 5x5, fp32 coefficients: one wavefront per SIMD
    (29, 36, 3, 1, 90, 5, "f32", "f16", 1),     # ... one channel, x3, fp16 image
    (33, 48, 4, 3, 128, 5, "f8", "f32", 1),     # ... 8-bit coefficients
    (30, 36, 2, 1, 75, 5, "f8", "f16", 2),      # ... one channel, x2, fp16 image
    (33, 47, 4, 3, 128, 5, "f16", "f32", 2),    # 128 atoms of 5x5: two pixels per lane
    (29, 36, 3, 1, 100, 5, "f16", "f16", 1),    # ... one channel, x3, fp16 image
    (26, 31, 2, 3, 73, 5, "bf16", "f32", 1),    # ... bfloat16, x2, HR width 62
    (40, 67, 4, 3, 128, 5, "bf16", "f32", 1),   # ... HR width 268, several tiles
    (33, 47, 4, 3, 72, 5, "bf16", "f32", 2),    # bfloat16 coefficients on the matrix-core path
    (29, 36, 3, 1, 72, 5, "bf16", "f16", 1),    # ... one channel, fp16 image, x3
    (17, 34, 4, 3, 7, 5, "bf16", "f32", 1),     # ... the 8-atom instantiation
    (30, 41, 2, 3, 30, 5, "bf16", "f32", 1),    # ... the 32-atom instantiation, x2
    (26, 31, 2, 3, 50, 5, "bf16", "f32", 1),    # ... HR width 62: generic kernel only
    (12, 20, 4, 3, 100, 7, "bf16", "f16", 1),   # ... 7x7 atoms, the 128-atom instantiation
    (22, 36, 3, 3, 60, 7, "bf16", "f32", 1),    # ... the 72-atom instantiation, x3
    (23, 35, 4, 3, 72, 3, "bf16", "f32", 1),    # ... 3x3 atoms
    (24, 36, 3, 1, 20, 3, "bf16", "f16", 1),    # ... one channel, x3, fp16 image
    (30, 41, 4, 2, 72, 5, "bf16", "f32", 1),    # ... two channels
    (30, 41, 2, 4, 20, 5, "bf16", "f16", 2),    # ... four channels, 32-atom instantiation
    (22, 36, 4, 1, 128, 7, "bf16", "f32", 1),   # ... 7x7, one channel
    (37, 53, 3, 3, 72, 5, "bf16", "f32", 1),    # ... HR width 159: the shifted last tile column
    (29, 35, 4, 1, 40, 5, "f8", "f16", 2),      # 8-bit coefficients, fp16 images of 1015 elements: the second starts mid-word
    (13, 15, 4, 3, 72, 5, "f8", "f16", 4),      # ... 585 elements each, four images
    (33, 47, 4, 3, 72, 5, "f8", "f32", 2),      # 8-bit E4M3 coefficients on the matrix-core path
    (29, 36, 3, 1, 72, 5, "f8", "f16", 1),      # ... one channel, fp16 image, x3
    (17, 34, 4, 3, 7, 5, "f8", "f32", 1),       # ... few atoms (the 8-atom instantiation)
    (26, 31, 2, 3, 50, 5, "f8", "f32", 1),      # ... HR width 62: generic kernel only
    (12, 20, 4, 3, 100, 7, "f8", "f16", 1),     # ... 7x7 atoms: the 128-atom instantiation (one wavefront per SIMD)
    (35, 49, 4, 3, 128, 7, "f8", "f16", 2),     # ... several tiles, two images
    (22, 36, 3, 1, 60, 7, "f8", "f32", 1),      # ... one channel, 72-atom instantiation, x3
    (26, 30, 2, 3, 72, 7, "f8", "f32", 1),      # ... x2
    (20, 24, 4, 3, 12, 7, "f8", "f32", 1),      # ... few atoms: generic kernel
    (22, 37, 4, 3, 128, 7, "f32", "f32", 2),    # fp32 coefficients, 7x7: the 128-atom instantiation (one wavefront per SIMD)
    (19, 30, 2, 3, 72, 7, "f32", "f16", 1),     # ... 72 atoms, fp16 image
    (27, 21, 3, 1, 100, 7, "f32", "f32", 1),    # ... one channel
    (20, 28, 4, 1, 60, 7, "f32", "f32", 1),     # ... one channel, 72-atom instantiation
    (16, 40, 4, 3, 11, 7, "f32", "f32", 1),     # ... few atoms: left to the generic kernel
    (24, 33, 4, 1, 9, 7, "f16", "f32", 1),      # 7x7, one channel, few atoms (16-atom instantiation)
    (24, 33, 4, 1, 70, 7, "f16", "f16", 1),     # ... 72-atom instantiation
    (30, 41, 4, 1, 8, 5, "f32", "f32", 1),      # 5x5, one channel, fp32 coefficients, 8-atom instantiation
    (30, 41, 4, 1, 30, 5, "f8", "f32", 1),      # ... 8-bit coefficients, 32-atom instantiation
    (30, 41, 4, 3, 44, 5, "f8", "f32", 1),      # 8-bit coefficients, 48-atom instantiation
    (33, 47, 4, 3, 72, 3, "f16", "f32", 2),     # 3x3 atoms on the matrix-core path
    (29, 38, 2, 3, 72, 3, "f16", "f16", 1),     # ... x2, fp16 image
    (27, 36, 3, 1, 30, 3, "f16", "f32", 1),     # ... one channel, 32-atom instantiation
    (21, 30, 4, 3, 6, 3, "f16", "f32", 1),      # ... 8-atom instantiation
    (25, 33, 2, 3, 72, 3, "f32", "f32", 1),     # ... fp32 coefficients, HR width 66
    (18, 26, 4, 1, 50, 3, "f32", "f16", 1),     # ... one channel
    (23, 35, 4, 3, 72, 3, "f8", "f32", 1),      # ... 8-bit coefficients
    (23, 35, 3, 1, 20, 3, "f8", "f16", 1),      # ... one channel, x3 (HR width 105: generic kernel only)
    (24, 36, 3, 1, 20, 3, "f8", "f16", 1),      # ... HR width 108
    (21, 30, 4, 3, 8, 3, "f32", "f32", 1),      # ... fp32 coefficients, 8-atom instantiation
    (21, 30, 4, 1, 5, 3, "f8", "f32", 1),       # ... 8-bit coefficients, 8-atom instantiation
    (41, 67, 3, 3, 72, 5, "f16", "f32", 2),     # HR width 201: rows start at odd element offsets, last tile column moved left
    (40, 43, 3, 3, 72, 5, "f16", "f16", 1),     # HR width 129: one column more than a tile, fp16 image
    (33, 49, 3, 3, 128, 7, "f16", "f16", 1),    # HR width 147, 7x7 (groups of two pixels)
    (29, 45, 3, 1, 72, 5, "f32", "f32", 1),     # HR width 135, fp32 coefficients
    (37, 53, 3, 3, 72, 5, "f8", "f32", 1),      # HR width 159, 8-bit coefficients: rows at odd byte offsets
    (18, 2, 3, 3, 72, 5, "f16", "f32", 1),      # HR width 6: generic kernel only
    (20, 65, 2, 3, 8, 5, "f16", "f32", 1),      # HR width 130, 8 atoms (tile 64 wide)
    (20, 64, 2, 3, 72, 5, "f16", "f32", 1),     # HR width 128: exactly one tile
    (22, 43, 3, 3, 72, 3, "f16", "f32", 2),     # HR width 129, 3x3
    (33, 47, 4, 4, 72, 5, "f16", "f32", 1),     # four channels on the matrix-core path (tile 128 x 8)
    (27, 45, 3, 4, 30, 5, "f16", "f16", 2),     # ... 32-atom instantiation, fp16 image, ragged width 135
    (29, 38, 2, 2, 72, 5, "f16", "f32", 1),     # two channels
    (31, 40, 4, 2, 17, 5, "f16", "f16", 1),     # ... 32-atom instantiation
    (20, 30, 4, 4, 72, 5, "f32", "f32", 1),     # four channels, fp32 coefficients: generic kernel only
]


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("case", RAGGED, ids=lambda c: "h%dw%ds%dC%dL%dk%d%s%sN%d" % c)
def test_ragged_shapes(oracle, case, kernel):
    h, w, s, C, L, k, cd, io, N = case
    wl = sr_synth.Workload("ragged", 7, N, C, h, w, s, L, k, cd, io, 0.0, 1.5)
    check_full(oracle, wl, kernel)


# ---- frames large enough for the big default tiles, with ragged tails ------------
# (the default tile grows with the frame: these sizes are past the thresholds)
BIG_RAGGED = [
    # (h, w, scale, C, L, k, coeff dtype, io dtype, N)
    (331, 501, 4, 3, 72, 5, "f16", "f32", 1),   # 1324 x 2004 = 2.65 Mpixel: 128 x 24 tiles, 55 rows + 4, 15 columns + 84
    (233, 267, 3, 3, 72, 5, "f16", "f32", 1),   # 699 x 801: 128 x 16 tiles at x3, odd width
    (150, 170, 4, 3, 72, 5, "f16", "f16", 1),   # 600 x 680 = 0.41 Mpixel at x4: 64 x 16 tiles
    (171, 151, 4, 3, 72, 5, "f8", "f32", 1),    # 684 x 604: 128 x 24 tiles, 8-bit coefficients
    (171, 151, 4, 3, 72, 5, "bf16", "f32", 1),  # ... bfloat16 coefficients
    (130, 200, 3, 1, 72, 5, "bf16", "f16", 1),  # ... 128 x 16 tiles, one channel
    (200, 191, 4, 3, 72, 5, "f32", "f32", 1),   # 800 x 764 = 0.61 Mpixel: 64 x 32 tiles, fp32 coefficients
    (181, 240, 4, 3, 8, 5, "f16", "f32", 1),    # 8 atoms: 64 x 32 tiles at three workgroups per CU
    (121, 163, 4, 3, 128, 7, "f16", "f16", 2),  # 7x7: 64 x 24 tiles
]


@pytest.mark.parametrize("case", BIG_RAGGED, ids=lambda c: "h%dw%ds%dC%dL%dk%d%s%sN%d" % c)
def test_big_default_tiles_with_ragged_tails(oracle, case):
    h, w, s, C, L, k, cd, io, N = case
    wl = sr_synth.Workload("bigragged", 8, N, C, h, w, s, L, k, cd, io, 0.0, 1.5)
    check_full(oracle, wl, MFMA)


# ---- dictionary-selective form -------------------------------------------------
@pytest.mark.parametrize("kernel", KERNELS)
def test_selective_kept_list_with_and_without_gamma(oracle, kernel):
    wl = sr_synth.scaled(sr_synth.WORKLOADS["4k_selective"], h=60, w=104)
    inp = sr_synth.make_inputs(wl, DEV)
    kept = inp["kept"]
    assert len(kept) == 8
    check_full(oracle, wl, kernel, kept=kept, inp=inp)
    gamma = np.linspace(0.5, 1.75, 8).astype(np.float32)
    check_full(oracle, wl, kernel, kept=kept[::-1].copy(), gamma=gamma, inp=inp)
    # an unordered list of odd length, and the full list in reverse
    check_full(oracle, wl, kernel, kept=np.array([70, 3, 41, 8, 0, 19, 5, 66, 23, 71, 12]), inp=inp)
    check_full(oracle, wl, kernel, kept=np.arange(71, -1, -1), inp=inp)


@pytest.mark.parametrize("cd", ["f16", "f32", "f8", "bf16"])
def test_kept_lists_around_every_built_capacity(oracle, cd):
    """The matrix-core kernel is built for 8/16/32/48/72 atoms (fewer sizes for some
    storage types); a kept list runs in the smallest one that holds it.  Lists one
    below, at and one above each size, with scales, against the oracle."""
    wl = sr_synth.Workload("capacity", 11, 1, 3, 20, 36, 4, 72, 5, cd, "f32", 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    rng = np.random.default_rng(5)
    for n_keep in (1, 7, 8, 9, 15, 16, 17, 31, 32, 33, 47, 48, 49, 71, 72):
        kept = rng.permutation(72)[:n_keep].astype(np.int32)
        gamma = rng.uniform(0.5, 1.5, size=n_keep).astype(np.float32)
        assert planned(inp, wl, MFMA, kept) == MFMA
        check_full(oracle, wl, MFMA, kept=kept, gamma=gamma, inp=inp)


# ---- arbitrary real coefficients: negative, unnormalised, fp16 subnormal ---------
@pytest.mark.parametrize("kernel", KERNELS)
def test_unnormalised_negative_and_subnormal_coefficients(oracle, kernel):
    wl = sr_synth.Workload("wild", 9, 1, 3, 24, 32, 4, 72, 5, "f16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(99)
    c = torch.randn(inp["coeff"].shape, generator=g, device=DEV)
    c[:, ::3] *= 3e-5                      # lands in the fp16 subnormal range
    c[:, 1::3] *= 0.05
    inp["coeff"] = c.to(torch.float16)
    assert int(((inp["coeff"].abs() < 6.1e-5) & (inp["coeff"] != 0)).sum()) > 1000
    check_full(oracle, wl, kernel, inp=inp)


@pytest.mark.parametrize("kernel", KERNELS)
def test_subnormal_only_coefficients_are_not_flushed(oracle, kernel):
    """All coefficients subnormal in fp16, dictionary scaled up so the exact
    result is O(1): a path that flushed subnormals would return zeros."""
    wl = sr_synth.Workload("subn", 10, 1, 3, 8, 16, 4, 72, 5, "f16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    inp["coeff"] = (inp["coeff"].float() * 2e-3).clamp(max=6.0e-5).to(torch.float16)
    assert float(inp["coeff"].abs().max()) < 6.1e-5      # every stored value is subnormal
    inp["dict"] = inp["dict"] * 500.0
    worst = check_full(oracle, wl, kernel, inp=inp)
    got = run_gpu(inp, wl, kernel).cpu().numpy()
    assert np.abs(got).mean() > 0.2, "output collapsed: subnormals were flushed"
    assert worst < 2e-3


@pytest.mark.parametrize("cd,io", [("f16", "f32"), ("f16", "f16"), ("f32", "f32"), ("f8", "f32"), ("bf16", "f32")])
def test_tensors_that_start_off_a_16_byte_boundary(oracle, cd, io):
    """Coefficients and output that start one element into their buffers (a slice of a
    larger allocation): the matrix-core kernel takes them, same values."""
    wl = sr_synth.Workload("offset", 14, 1, 3, 30, 41, 4, 72, 5, cd, io, 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    cbuf = torch.empty((inp["coeff"].numel() + 1,), device=DEV, dtype=inp["coeff"].dtype)
    cview = cbuf[1:].view(inp["coeff"].shape)
    cview.copy_(inp["coeff"])
    obuf = torch.full((wl.n * wl.c * wl.H * wl.W + 1,), float("nan"), device=DEV, dtype=inp["lr"].dtype)
    oview = obuf[1:].view(wl.n, wl.c, wl.H, wl.W)
    opts = sr.make_options(MFMA, 0)
    assert sr.sr_dict_assemble_plan(inp["lr"], cview, inp["dict"], wl.L, wl.k, wl.scale, wl.c, oview, opts=opts) == MFMA
    sr.sr_dict_assemble_ex(inp["lr"], cview, inp["dict"], wl.L, wl.k, wl.scale, wl.c, oview, opts=opts)
    torch.cuda.synchronize()
    assert torch.isnan(obuf[0])
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale)
    worst, tol, ok = tolerance_ok(oview.float().cpu().numpy(), ref, cd, io == "f16")
    assert ok, f"worst error {worst:.3e} exceeds {tol:.0e}"
    assert torch.equal(oview, run_gpu(inp, wl, MFMA))


# ---- stage 1 alone, and the delta-atom identity -----------------------------------
@pytest.mark.parametrize("scale", [2, 3, 4])
@pytest.mark.parametrize("io", ["f32", "f16"])
@pytest.mark.parametrize("w", [53, 52, 1, 130])     # HR widths with and without whole groups of four pixels
def test_bicubic_entry_point(oracle, scale, io, w):
    wl = sr_synth.Workload("bic", 11, 2, 3, 37, w, scale, 1, 3, "f32", io)
    lr = sr_synth.make_lr(wl, DEV)
    out = torch.full((wl.n, wl.c, wl.H, wl.W), float("nan"), device=DEV, dtype=torch.float32)
    sr.sr_bicubic_upsample(lr, scale, wl.c, out)
    torch.cuda.synchronize()
    ref = oracle.bicubic(lr.cpu().numpy(), scale)
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-5 * np.maximum(1.0, np.abs(ref)))
    # an output that starts 4 bytes off a 16-byte boundary: same values
    buf = torch.full((out.numel() + 1,), float("nan"), device=DEV, dtype=torch.float32)
    shifted = buf[1:].view(out.shape)
    sr.sr_bicubic_upsample(lr, scale, wl.c, shifted)
    torch.cuda.synchronize()
    assert torch.equal(shifted, out) and torch.isnan(buf[0])
    if io == "f16":
        out16 = torch.empty_like(out, dtype=torch.float16)
        sr.sr_bicubic_upsample(lr, scale, wl.c, out16)
        torch.cuda.synchronize()
        assert torch.equal(out16, out.to(torch.float16))
        buf16 = torch.zeros((out.numel() + 1,), device=DEV, dtype=torch.float16)
        sr.sr_bicubic_upsample(lr, scale, wl.c, buf16[1:].view(out.shape))
        torch.cuda.synchronize()
        assert torch.equal(buf16[1:].view(out.shape), out16) and float(buf16[0]) == 0.0


def test_bicubic_entry_point_random_shapes(oracle):
    """Frames smaller and larger than the 256 x 16 pixels of a workgroup, ragged in both directions."""
    rng = np.random.default_rng(2024)
    cases = [(1, 1, 1, 1, 2), (1, 1, 1, 2, 3), (1, 2, 2, 1, 4), (1, 1, 3, 400, 2), (2, 1, 50, 3, 4)]
    while len(cases) < 30:
        cases.append((int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 45)),
                      int(rng.integers(1, 330)), int(rng.integers(2, 5))))
    for i, (n, c, h, w, scale) in enumerate(cases):
        io = "f16" if i % 3 == 2 else "f32"
        wl = sr_synth.Workload("bicr", 40 + i, n, c, h, w, scale, 1, 3, "f32", io)
        lr = sr_synth.make_lr(wl, DEV)
        out = torch.full((n, c, wl.H, wl.W), float("nan"), device=DEV, dtype=torch.float32)
        sr.sr_bicubic_upsample(lr, scale, c, out)
        torch.cuda.synchronize()
        ref = oracle.bicubic(lr.cpu().numpy(), scale)
        got = out.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref) <= 1e-5 * np.maximum(1.0, np.abs(ref))), (n, c, h, w, scale, io)


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("scale,k", [(2, 5), (3, 5), (4, 5), (4, 7), (3, 3)])
def test_centred_delta_atom_equals_bicubic_bit_for_bit(kernel, scale, k):
    wl = sr_synth.Workload("delta", 12, 1, 3, 23, 34, scale, 8, k, "f16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    D = torch.randn_like(inp["dict"])
    D[5] = 0
    D[5, k // 2, k // 2] = 1.0
    inp["dict"] = D
    coeff = torch.zeros_like(inp["coeff"])
    coeff[:, 5] = 1.0
    inp["coeff"] = coeff
    if planned(inp, wl, kernel) != kernel:
        pytest.skip("this kernel does not take this case")
    got = run_gpu(inp, wl, kernel)
    bic = torch.empty_like(got)
    sr.sr_bicubic_upsample(inp["lr"], scale, wl.c, bic)
    torch.cuda.synchronize()
    assert torch.equal(got, bic)


@pytest.mark.parametrize("kernel", KERNELS)
def test_off_centre_delta_atoms_on_gpu(oracle, kernel):
    """Orientation and border clamp of the patch, with deltas in each corner."""
    wl = sr_synth.Workload("corner", 13, 1, 1, 10, 18, 4, 8, 5, "f16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    D = torch.zeros_like(inp["dict"])
    for l, (dy, dx) in enumerate([(0, 0), (0, 4), (4, 0), (4, 4), (1, 3), (3, 1), (2, 0), (0, 2)]):
        D[l, dy, dx] = 1.0
    inp["dict"] = D
    check_full(oracle, wl, kernel, inp=inp)


@pytest.mark.parametrize("kernel", KERNELS)
def test_constant_image_is_preserved(kernel):
    wl = sr_synth.Workload("const", 14, 1, 3, 20, 24, 4, 72, 5, "f16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    inp["lr"] = torch.full_like(inp["lr"], 0.625)
    if planned(inp, wl, kernel) != kernel:
        pytest.skip("this kernel does not take this case")
    got = run_gpu(inp, wl, kernel)
    assert float((got - 0.625).abs().max()) < 2e-3


def test_empty_batch_and_error_statuses_on_device():
    wl = sr_synth.Workload("empty", 15, 0, 3, 8, 8, 2, 4, 3, "f32", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    out = torch.empty((0, 3, 16, 16), device=DEV)
    sr.sr_dict_assemble(inp["lr"], inp["coeff"], inp["dict"], 4, 3, 2, 3, out)
    wl = sr_synth.scaled(wl, n=1)
    inp = sr_synth.make_inputs(wl, DEV)
    out = torch.zeros((1, 3, 16, 16), device=DEV)
    with pytest.raises(sr.SrError) as e:
        sr.sr_dict_assemble(inp["lr"], inp["coeff"], inp["dict"], 4, 3, 3, 3, out)
    assert e.value.status == -2
    with pytest.raises(sr.SrError) as e:
        sr.sr_dict_assemble_selective(inp["lr"], inp["coeff"], inp["dict"], 4, 3, 2, 3, out, kept=[1, 1])
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert not out.any()      # nothing was written by the failed calls


def test_runs_on_a_side_stream():
    wl = sr_synth.scaled(sr_synth.WORKLOADS["tiny"])
    inp = sr_synth.make_inputs(wl, DEV)
    a = run_gpu(inp, wl, sr.SR_KERNEL_AUTO)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    b = torch.empty_like(a)
    with torch.cuda.stream(st):
        sr.sr_dict_assemble(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, b, stream=st)
    st.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("kernel", KERNELS)
def test_replays_inside_a_captured_graph(kernel):
    """The library allocates nothing and enqueues one kernel, so a call can be captured
    in a HIP graph.  Three replays, new inputs copied into the captured buffers between
    them and eager work in between, each compared with an eager call."""
    wl = sr_synth.scaled(sr_synth.WORKLOADS["4k_dense"], h=40, w=64)
    first = sr_synth.make_inputs(wl, DEV)
    if planned(first, wl, kernel) != kernel:
        pytest.skip("this kernel does not take this case")
    lr, coeff, D = first["lr"].clone(), first["coeff"].clone(), first["dict"].clone()
    out = torch.zeros((wl.n, wl.c, wl.H, wl.W), device=DEV)
    opts = sr.make_options(kernel, 0)
    sr.sr_dict_assemble_ex(lr, coeff, D, wl.L, wl.k, wl.scale, wl.c, out, opts=opts)   # warm-up outside capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sr.sr_dict_assemble_ex(lr, coeff, D, wl.L, wl.k, wl.scale, wl.c, out, opts=opts)
    for rep in range(3):
        fresh = sr_synth.make_inputs(sr_synth.scaled(wl, index=wl.index + 1 + rep), DEV)
        lr.copy_(fresh["lr"]); coeff.copy_(fresh["coeff"]); D.copy_(fresh["dict"])
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = run_gpu(fresh, wl, kernel)
        assert torch.equal(out, eager), f"replay {rep}"


def test_tile_sweep_returns_a_valid_shape():
    """The measured launch-shape search (stand-in for the paper's constrained
    Bayesian search) visits every built tile shape and picks one of them."""
    from paper_2303_08999_amd import tune
    wl = sr_synth.scaled(sr_synth.WORKLOADS["4k_dense"], h=96, w=128)
    inp = sr_synth.make_inputs(wl, DEV)
    out = torch.empty((wl.n, wl.c, wl.H, wl.W), device=DEV)
    res = tune.sweep_tiles(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, out, reps=3)
    assert [t for t, _ in res] == list(range(10))
    assert all(ms > 0 for _, ms in res)
    assert tune.best_tile(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, out, reps=3) in range(10)
    # every swept index is another launch shape (index 0 is the default: one of the nine)
    tiles = [sr.sr_dict_assemble_launch_shape(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, out,
                                              opts=sr.make_options(MFMA, t))[1] for t, _ in res]
    assert len(set(tiles[1:])) == 9 and tiles[0] in tiles[1:]
    # at scale 3 the 128 x 24 tile does not exist, and a family with one built shape sweeps index 0 only
    wl3 = sr_synth.scaled(wl, scale=3)
    i3 = sr_synth.make_inputs(wl3, DEV)
    o3 = torch.empty((wl3.n, wl3.c, wl3.H, wl3.W), device=DEV)
    assert [t for t, _ in tune.sweep_tiles(i3["lr"], i3["coeff"], i3["dict"], wl3.L, wl3.k, wl3.scale, wl3.c, o3, reps=1)] == [0, 1, 2, 3, 4, 5, 6, 8, 9]
    wl8 = sr_synth.scaled(wl, coeff_dtype="f8")
    i8 = sr_synth.make_inputs(wl8, DEV)
    assert [t for t, _ in tune.sweep_tiles(i8["lr"], i8["coeff"], i8["dict"], wl8.L, wl8.k, wl8.scale, wl8.c, out, reps=1)] == [0]
    # two channels, fp32 coefficients: the matrix-core kernel does not apply, nothing to sweep
    wl32 = sr_synth.scaled(sr_synth.WORKLOADS["tiny"], c=2)
    i32 = sr_synth.make_inputs(wl32, DEV)
    o32 = torch.empty((1, wl32.c, wl32.H, wl32.W), device=DEV)
    assert tune.sweep_tiles(i32["lr"], i32["coeff"], i32["dict"], wl32.L, wl32.k, wl32.scale, wl32.c, o32) == []
