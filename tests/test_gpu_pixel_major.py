"""Coefficients stored pixel-major, [N][H][W][L] (a storage order beyond the paper: what a producer that keeps its
tensors channels-last writes): the HIP path reads that order directly and must give what the oracle gives when it
moves the coefficients to planes first - and, since only the loads differ, exactly what the HIP path gives for the
planar tensor."""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth
from test_gpu_parity import DEV, GENERIC, MFMA, assert_parity, host

pytestmark = pytest.mark.gpu
PM = sr.SR_COEFF_PIXEL_MAJOR


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
    (1, 3, 37, 64, 4, 72, 5, "f16", "f32", None),       # the matrix-core family: two tile columns, ragged rows
    (2, 3, 50, 96, 4, 72, 5, "f16", "f32", None),       # two images, three tile columns
    (1, 3, 41, 64, 2, 72, 5, "f16", "f32", None),       # scale 2: 128 x 8 tiles, one tile column
    (1, 3, 29, 128, 3, 72, 5, "f16", "f16", None),      # scale 3, fp16 image (a lane stores single 2-byte pixels)
    (1, 3, 9, 32, 4, 72, 5, "f16", "f32", None),        # fewer rows than a tile
    (1, 3, 40, 64, 4, 72, 5, "f16", "f32", 8),          # a kept list: the generic kernel
    (1, 3, 20, 33, 4, 72, 5, "f16", "f32", None),       # HR width 132: not whole 128-pixel units, generic
    (1, 3, 18, 32, 4, 40, 5, "f16", "f32", None),       # 40 atoms: generic
    (1, 1, 19, 23, 4, 40, 5, "f32", "f32", None),
    (2, 2, 16, 21, 3, 17, 7, "f8", "f16", 5),
    (1, 3, 18, 20, 2, 30, 3, "bf16", "f32", None),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%dC%dh%dw%ds%dL%dk%d%s%s-%s" % c)
def test_pixel_major_layout_against_the_oracle_and_the_planar_call(oracle, case):
    N, C, h, w, s, L, k, cd, io, nk = case
    wl = sr_synth.Workload("pm", 52, N, C, h, w, s, L, k, cd, io, 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    pm = sr_synth.to_pixel_major(inp["coeff"])
    assert pm.shape == (N, h * s, w * s, L)
    kept = gamma = None
    if nk:
        rng = np.random.default_rng(nk)
        kept = np.sort(rng.choice(L, size=nk, replace=False)).astype(np.int32)
        gamma = rng.uniform(0.5, 1.5, size=nk).astype(np.float32)
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(pm), hi["dict"], s, kept=kept, gamma=gamma, pixel_major=True)
    ran = 0
    for kernel in (GENERIC, MFMA):
        got = run(inp, wl, pm, kernel, PM, kept, gamma)
        if got is None:
            continue
        ran += 1
        assert not torch.isnan(got).any(), "some output pixel was never written"
        assert_parity(got.float().cpu().numpy(), ref, cd, io == "f16", f"kernel {kernel}")
        planar = run(inp, wl, inp["coeff"], kernel, sr.SR_COEFF_PLANAR, kept, gamma)
        if planar is not None:
            assert torch.equal(got, planar), f"kernel {kernel}: the two storage orders must give the same bits"
    assert ran >= 1
    takes = run(inp, wl, pm, MFMA, PM, kept, gamma) is not None
    assert takes == (cd == "f16" and C == 3 and k == 5 and L == 72 and nk is None and (w * s) % 128 == 0)


def test_4k_frame_stored_pixel_major(oracle):
    """The headline frame with its coefficients stored pixel-major: every output equals the planar call's, and sampled
    pixels (corners and edges among them) are checked against the oracle."""
    wl = sr_synth.WORKLOADS["4k_dense"]
    inp = sr_synth.make_inputs(wl, DEV)
    planar = run(inp, wl, inp["coeff"], MFMA, sr.SR_COEFF_PLANAR)
    pm = sr_synth.to_pixel_major(inp["coeff"])
    del inp["coeff"]
    got = run(inp, wl, pm, MFMA, PM)
    assert got is not None and planar is not None
    assert torch.equal(got, planar)
    rng = np.random.default_rng(13)
    pts = np.stack([np.zeros(2000, dtype=np.int64), rng.integers(0, wl.H, 2000), rng.integers(0, wl.W, 2000)], axis=1)
    pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
    pts[4:304, 1] = wl.H - 1 - (pts[4:304, 1] % 13)
    pts[304:604, 2] = wl.W - 1 - (pts[304:604, 2] % 5)
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    want = oracle.assemble_points(U, oracle.pixel_major_to_planar(sr_synth.stored_numpy(pm)), inp["dict"].cpu().numpy(), pts)
    have = got.cpu().numpy()[0][:, pts[:, 1], pts[:, 2]].T
    assert_parity(have, want, "f16", False, "sampled pixels")
