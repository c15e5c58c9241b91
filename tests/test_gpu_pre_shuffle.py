"""Coefficients in the layout they have BEFORE the coefficient network's pixel-shuffle layer
(section II-B, stage 2), [N][L*s*s][h][w]: the HIP path reads that layout directly and must give
what the oracle gives when it applies the pixel-shuffle first - and, since only the loads differ,
exactly what the HIP path gives for the shuffled tensor."""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth
from test_gpu_parity import DEV, GENERIC, MFMA, assert_parity, host

pytestmark = pytest.mark.gpu


def run(inp, wl, coeff, kernel, layout, kept=None, gamma=None):
    out = torch.full((wl.n, wl.c, wl.H, wl.W), float("nan"), device=DEV, dtype=inp["lr"].dtype)
    opts = sr.make_options(kernel, 0, layout)
    if sr.sr_dict_assemble_plan(inp["lr"], coeff, inp["dict"], wl.L, wl.k, wl.scale, wl.c, out, kept=kept, opts=opts) != kernel:
        return None
    sr.sr_dict_assemble_ex(inp["lr"], coeff, inp["dict"], wl.L, wl.k, wl.scale, wl.c, out, kept=kept, gamma=gamma, opts=opts)
    torch.cuda.synchronize()
    return out


CASES = [
    # (N, C, h, w, scale, L, k, coeff dtype, image dtype, kept atoms or None)
    (1, 3, 37, 64, 4, 72, 5, "f16", "f32", None),       # the matrix-core family: several tiles, ragged rows
    (2, 3, 50, 96, 4, 72, 5, "f16", "f32", None),       # two images, 384 wide: a full and a partial 256-pixel tile column
    (2, 3, 21, 72, 4, 72, 5, "f16", "f16", None),       # scale 4 with an fp16 image (a lane stores four pixels as 8 bytes)
    (1, 3, 33, 132, 4, 72, 5, "f16", "f32", 8),         # scale 4, the small capacity, three tile columns, rows not a multiple of 8
    (1, 3, 9, 4, 4, 72, 5, "f16", "f32", None),         # scale 4, one LR pixel group wide: one lane pair per row does the work
    (1, 3, 27, 140, 2, 72, 5, "f16", "f16", 70),        # scale 2, fp16 image, 70 kept atoms with gamma
    (1, 3, 41, 66, 2, 72, 5, "f16", "f32", None),       # scale 2: a lane's four pixels span two LR columns
    (1, 3, 29, 44, 3, 72, 5, "f16", "f32", None),       # scale 3, LR width a multiple of 4: 384-pixel rows in three units
    (2, 3, 20, 260, 3, 72, 5, "f16", "f32", None),      # scale 3, two images, 780 wide: two full tile columns and 12 pixels
    (1, 3, 30, 132, 3, 72, 5, "f16", "f16", 8),         # scale 3, fp16 image, the small capacity
    (1, 3, 40, 64, 4, 72, 5, "f16", "f32", 8),          # a kept list of 8: the small capacity
    (1, 3, 33, 48, 3, 72, 5, "f16", "f16", 66),         # fp16 image, 66 kept atoms with gamma
    (1, 3, 20, 33, 4, 72, 5, "f16", "f32", None),       # HR width 132: not whole tiles
    (1, 1, 19, 23, 4, 40, 5, "f32", "f32", None),       # everything else runs on the generic kernel
    (2, 2, 16, 21, 3, 17, 7, "f8", "f16", 5),
    (1, 3, 18, 20, 2, 30, 3, "bf16", "f32", None),
    (1, 3, 37, 64, 4, 72, 5, "bf16", "f32", None),      # bfloat16 coefficients in the permuted-slot forms: scale 4,
    (2, 3, 29, 44, 3, 72, 5, "bf16", "f32", None),      #   scale 3,
    (1, 3, 41, 68, 2, 72, 5, "bf16", "f16", 70),        #   scale 2 with 70 kept atoms and an fp16 image
    (1, 3, 20, 30, 4, 72, 5, "bf16", "f32", None),      # bfloat16, LR width not a multiple of 4: the generic kernel
    (1, 3, 15, 17, 3, 72, 5, "f16", "f32", None),       # HR width 51: not whole pixel groups
    (1, 3, 23, 18, 3, 72, 5, "f16", "f32", None),       # scale 3, LR width not a multiple of 4: one 16-bit load per pixel and plane
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%dC%dh%dw%ds%dL%dk%d%s%s-%s" % c)
def test_pre_shuffle_layout_against_the_oracle_and_the_planar_call(oracle, case):
    N, C, h, w, s, L, k, cd, io, nk = case
    wl = sr_synth.Workload("ps", 50, N, C, h, w, s, L, k, cd, io, 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    pre = sr_synth.to_pre_shuffle(inp["coeff"], s)
    assert pre.shape == (N, L * s * s, h, w)
    kept = gamma = None
    if nk:
        rng = np.random.default_rng(nk)
        kept = np.sort(rng.choice(L, size=nk, replace=False)).astype(np.int32)
        gamma = rng.uniform(0.5, 1.5, size=nk).astype(np.float32)
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(pre), hi["dict"], s, kept=kept, gamma=gamma, pre_shuffle=True)
    ran = 0
    for kernel in (GENERIC, MFMA):
        got = run(inp, wl, pre, kernel, sr.SR_COEFF_PRE_SHUFFLE, kept, gamma)
        if got is None:
            continue
        ran += 1
        assert not torch.isnan(got).any(), "some output pixel was never written"
        assert_parity(got.float().cpu().numpy(), ref, cd, io == "f16", f"kernel {kernel}")
        planar = run(inp, wl, inp["coeff"], kernel, sr.SR_COEFF_PLANAR, kept, gamma)
        if planar is not None:
            assert torch.equal(got, planar), f"kernel {kernel}: the two layouts must give the same bits"
    assert ran >= 1
    if cd == "f16" and C == 3 and k == 5 and (h * s) and (w * s) % 4 == 0 and (nk is None or nk <= 8 or nk >= 65):
        assert run(inp, wl, pre, MFMA, sr.SR_COEFF_PRE_SHUFFLE, kept, gamma) is not None, "this case belongs to the matrix-core kernel"
    if cd == "bf16" and C == 3 and k == 5:
        takes = run(inp, wl, pre, MFMA, sr.SR_COEFF_PRE_SHUFFLE, kept, gamma) is not None
        assert takes == (w % 4 == 0 and (nk is None or nk >= 65)), "bfloat16: the permuted-slot forms only"


def test_4k_frame_in_the_pre_shuffle_layout(oracle):
    """The headline frame handed over as the network's 1152-channel LR tensor: every output equals the
    planar call's, and sampled pixels (corners and edges among them) are checked against the oracle,
    which shuffles first."""
    wl = sr_synth.WORKLOADS["4k_dense"]
    inp = sr_synth.make_inputs(wl, DEV)
    planar = run(inp, wl, inp["coeff"], sr.SR_KERNEL_AUTO if False else MFMA, sr.SR_COEFF_PLANAR)
    pre = sr_synth.to_pre_shuffle(inp["coeff"], wl.scale)
    host_pre = sr_synth.stored_numpy(pre)
    del inp["coeff"]
    got = run(inp, wl, pre, MFMA, sr.SR_COEFF_PRE_SHUFFLE)
    assert got is not None and planar is not None
    assert torch.equal(got, planar)
    rng = np.random.default_rng(12)
    pts = np.stack([np.zeros(3000, dtype=np.int64), rng.integers(0, wl.H, 3000), rng.integers(0, wl.W, 3000)], axis=1)
    pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
    pts[4:504, 1] = wl.H - 1 - (pts[4:504, 1] % 13)
    pts[504:1004, 2] = wl.W - 1 - (pts[504:1004, 2] % 5)
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    want = oracle.assemble_points(U, oracle.pixel_shuffle(host_pre, wl.scale), inp["dict"].cpu().numpy(), pts)
    have = got.cpu().numpy()[0][:, pts[:, 1], pts[:, 2]].T
    assert_parity(have, want, "f16", False, "sampled pixels")


def test_1080p_x3_frame_in_the_pre_shuffle_layout():
    """The 1080p x3 workload (384-pixel rows in three units, one workgroup of eight wavefronts per CU) equals the
    planar call bit for bit; the planar call itself is checked against the oracle in test_gpu_parity.py."""
    wl = sr_synth.WORKLOADS["1080p_fp16"]
    inp = sr_synth.make_inputs(wl, DEV)
    planar = run(inp, wl, inp["coeff"], MFMA, sr.SR_COEFF_PLANAR)
    got = run(inp, wl, sr_synth.to_pre_shuffle(inp["coeff"], wl.scale), MFMA, sr.SR_COEFF_PRE_SHUFFLE)
    assert got is not None and planar is not None
    assert torch.equal(got, planar)


def test_random_shapes_in_the_pre_shuffle_layout():
    """Seeded random frames of the matrix-core family (5x5 atoms, three channels, fp16 coefficients, all 72 atoms or a
    kept list of up to 8): LR widths that are and are not multiples of 4, every scale, one to three images, fp16 and
    fp32 images.  Whatever form serves the case (permuted slots, or one 16-bit load per pixel), the output must be the
    planar call's, bit for bit, and every pixel must be written."""
    rng = np.random.default_rng(20230317)
    forms = 0
    for index in range(60):
        s = int(rng.choice([2, 3, 4]))
        h = int(rng.integers(1, 40))
        w = int(rng.integers(1, 30)) * 4 if rng.random() < 0.7 else int(rng.integers(2, 120))
        n = int(rng.choice([1, 1, 2, 3]))
        io = str(rng.choice(["f32", "f16"]))
        wl = sr_synth.Workload("psr", 300 + index, n, 3, h, w, s, 72, 5, "f16", io, 0.0, 1.5)
        kept = gamma = None
        if rng.random() < 0.4:
            nk = int(rng.integers(1, 9))
            kept = np.sort(rng.choice(72, size=nk, replace=False)).astype(np.int32)
            gamma = rng.uniform(0.5, 1.5, size=nk).astype(np.float32)
        inp = sr_synth.make_inputs(wl, DEV)
        planar = run(inp, wl, inp["coeff"], MFMA, sr.SR_COEFF_PLANAR, kept, gamma)
        got = run(inp, wl, sr_synth.to_pre_shuffle(inp["coeff"], s), MFMA, sr.SR_COEFF_PRE_SHUFFLE, kept, gamma)
        if planar is None or got is None:
            continue                                    # a width the matrix-core kernel does not take
        assert not torch.isnan(got).any(), f"{wl}: some output pixel was never written"
        assert torch.equal(got, planar), f"{wl} kept {kept}: the two layouts must give the same bits"
        forms += 1
    assert forms >= 40, forms


@pytest.mark.parametrize("scale", [2, 3, 4])
def test_pre_shuffle_call_replays_inside_a_captured_graph(scale):
    """The pre-shuffle forms, like the planar one, are one kernel with no allocation: three replays of a captured
    call with new inputs copied into the captured buffers, each compared with an eager call."""
    wl = sr_synth.Workload("psg", 65, 1, 3, 24, 64, scale, 72, 5, "f16", "f32", 0.0, 1.5)
    first = sr_synth.make_inputs(wl, DEV)
    lr, pre, D = first["lr"].clone(), sr_synth.to_pre_shuffle(first["coeff"], scale).clone(), first["dict"].clone()
    out = torch.zeros((wl.n, wl.c, wl.H, wl.W), device=DEV)
    opts = sr.make_options(MFMA, 0, sr.SR_COEFF_PRE_SHUFFLE)
    call = lambda: sr.sr_dict_assemble_ex(lr, pre, D, wl.L, wl.k, wl.scale, wl.c, out, opts=opts)
    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        fresh = sr_synth.make_inputs(sr_synth.scaled(wl, index=wl.index + 1 + rep), DEV)
        fp = sr_synth.to_pre_shuffle(fresh["coeff"], scale)
        lr.copy_(fresh["lr"]); pre.copy_(fp); D.copy_(fresh["dict"])
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = run(fresh, wl, fp, MFMA, sr.SR_COEFF_PRE_SHUFFLE)
        assert torch.equal(out, eager), f"replay {rep}"
