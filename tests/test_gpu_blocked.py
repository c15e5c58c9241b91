"""Coefficients stored blocked (SR_COEFF_BLOCKED: the order in which the matrix-core kernel consumes them; a storage order
beyond the paper): the HIP path reads that order directly and must give what the oracle gives when it moves the
coefficients to planes first - and, since only the loads differ, exactly what the HIP path gives for the planar tensor."""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth
from test_gpu_parity import DEV, GENERIC, MFMA, assert_parity, host

pytestmark = pytest.mark.gpu
BLK = sr.SR_COEFF_BLOCKED


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
    (1, 3, 41, 64, 2, 72, 5, "f16", "f32", None),       # scale 2: 128 x 16 tiles, one tile column
    (1, 3, 29, 128, 3, 72, 5, "f16", "f16", None),      # scale 3, fp16 image
    (1, 3, 9, 32, 4, 72, 5, "f16", "f32", None),        # fewer rows than a tile
    (3, 3, 1, 32, 4, 72, 5, "f16", "f32", None),        # one LR row, three images
    (1, 3, 37, 64, 4, 72, 5, "f8", "f32", None),        # 8-bit coefficients in the same order: the matrix-core family
    (2, 3, 29, 128, 3, 72, 5, "f8", "f16", None),
    (1, 3, 21, 64, 2, 72, 5, "f8", "f32", None),
    (1, 3, 37, 64, 4, 72, 5, "bf16", "f32", None),      # bfloat16 coefficients
    (1, 3, 29, 128, 3, 72, 5, "bf16", "f16", None),
    (1, 3, 40, 64, 4, 72, 5, "f16", "f32", 8),          # a kept list: the generic kernel
    (1, 3, 18, 32, 4, 40, 5, "f16", "f32", None),       # 40 atoms (two pieces and a last one): generic
    (1, 1, 19, 32, 4, 64, 5, "f32", "f32", None),       # 64 atoms: no last piece
    (2, 2, 16, 128, 3, 24, 7, "f8", "f16", 5),
    (1, 3, 18, 64, 2, 8, 3, "bf16", "f32", None),       # 8 atoms: the last piece only
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%dC%dh%dw%ds%dL%dk%d%s%s-%s" % c)
def test_blocked_layout_against_the_oracle_and_the_planar_call(oracle, case):
    N, C, h, w, s, L, k, cd, io, nk = case
    wl = sr_synth.Workload("blk", 58, N, C, h, w, s, L, k, cd, io, 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    blk = sr_synth.to_blocked(inp["coeff"])
    assert blk.shape == (N, h * s, w * s // 128, 128 * L)
    kept = gamma = None
    if nk:
        rng = np.random.default_rng(nk)
        kept = np.sort(rng.choice(L, size=nk, replace=False)).astype(np.int32)
        gamma = rng.uniform(0.5, 1.5, size=nk).astype(np.float32)
    hi = host(inp)
    ref = oracle.dict_assemble(hi["lr"], sr_synth.stored_numpy(blk), hi["dict"], s, kept=kept, gamma=gamma, blocked=True)
    ran = 0
    for kernel in (GENERIC, MFMA):
        got = run(inp, wl, blk, kernel, BLK, kept, gamma)
        if got is None:
            continue
        ran += 1
        assert not torch.isnan(got).any(), "some output pixel was never written"
        assert_parity(got.float().cpu().numpy(), ref, cd, io == "f16", f"kernel {kernel}")
        planar = run(inp, wl, inp["coeff"], kernel, sr.SR_COEFF_PLANAR, kept, gamma)
        if planar is not None:
            assert torch.equal(got, planar), f"kernel {kernel}: the two storage orders must give the same bits"
    assert ran >= 1
    takes = run(inp, wl, blk, MFMA, BLK, kept, gamma) is not None
    assert takes == (cd in ("f16", "f8", "bf16") and C == 3 and k == 5 and L == 72 and nk is None)


@pytest.mark.parametrize("name", ["4k_dense", "4k_dense_fp8"])
def test_4k_frame_stored_blocked(oracle, name):
    """The headline frame with its coefficients stored blocked: every output equals the planar call's, and sampled pixels
    (corners and edges among them) are checked against the oracle."""
    wl = sr_synth.WORKLOADS[name]
    inp = sr_synth.make_inputs(wl, DEV)
    planar = run(inp, wl, inp["coeff"], MFMA, sr.SR_COEFF_PLANAR)
    blk = sr_synth.to_blocked(inp["coeff"])
    del inp["coeff"]
    got = run(inp, wl, blk, MFMA, BLK)
    assert got is not None and planar is not None
    assert torch.equal(got, planar)
    rng = np.random.default_rng(15)
    pts = np.stack([np.zeros(2000, dtype=np.int64), rng.integers(0, wl.H, 2000), rng.integers(0, wl.W, 2000)], axis=1)
    pts[:4] = [(0, 0, 0), (0, wl.H - 1, wl.W - 1), (0, 0, wl.W - 1), (0, wl.H - 1, 0)]
    pts[4:304, 1] = wl.H - 1 - (pts[4:304, 1] % 13)
    pts[304:604, 2] = wl.W - 1 - (pts[304:604, 2] % 5)
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    want = oracle.assemble_points(U, oracle.blocked_to_planar(sr_synth.stored_numpy(blk)), inp["dict"].cpu().numpy(), pts)
    have = got.cpu().numpy()[0][:, pts[:, 1], pts[:, 2]].T
    assert_parity(have, want, wl.coeff_dtype, False, "sampled pixels")


@pytest.mark.parametrize("kind", ["values", "logits"])
def test_blocked_call_replays_inside_a_captured_graph(kind):
    """The blocked forms (stored coefficients and logits), with the kernel's L2 write-back pacing in them, are one kernel with
    no allocation: three replays of a captured call with new inputs copied into the captured buffers, each compared with an
    eager call.  The frame is large enough (several tiles per workgroup, a launch longer than the pacing period) for the
    write-back requests to fire."""
    wl = sr_synth.Workload("blg", 66, 2, 3, 270, 480, 4, 72, 5, "f16", "f32", 0.0, 1.5)
    make = sr_synth.make_logits if kind == "logits" else sr_synth.make_coeff
    first = sr_synth.make_inputs(wl, DEV)
    lr, blk, D = first["lr"].clone(), sr_synth.to_blocked(make(wl, DEV)).clone(), first["dict"].clone()
    out = torch.zeros((wl.n, wl.c, wl.H, wl.W), device=DEV)
    opts = sr.make_options(MFMA, 0, BLK, sr.SR_COEFF_LOGITS if kind == "logits" else sr.SR_COEFF_VALUES)
    call = lambda: sr.sr_dict_assemble_ex(lr, blk, D, wl.L, wl.k, wl.scale, wl.c, out, opts=opts)
    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        w2 = sr_synth.scaled(wl, index=wl.index + 1 + rep)
        fresh = sr_synth.make_inputs(w2, DEV)
        fb = sr_synth.to_blocked(make(w2, DEV))
        lr.copy_(fresh["lr"]); blk.copy_(fb); D.copy_(fresh["dict"])
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = torch.full_like(out, float("nan"))
        sr.sr_dict_assemble_ex(fresh["lr"], fb, fresh["dict"], wl.L, wl.k, wl.scale, wl.c, eager, opts=opts)
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep}"
