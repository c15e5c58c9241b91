"""Coefficients as per-pixel (atom index, value) lists - an extension beyond the paper - through the
C ABI against the oracle on the same stored lists."""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth
from test_gpu_parity import DEV, GENERIC, MFMA, parity_bound

pytestmark = pytest.mark.gpu


def run(inp, wl, idx, val, kernel=sr.SR_KERNEL_AUTO):
    """The call's output, or None if this kernel does not take the case."""
    out = torch.full((wl.n, wl.c, wl.H, wl.W), float("nan"), device=DEV, dtype=inp["lr"].dtype)
    try:
        sr.sr_dict_assemble_list_ex(inp["lr"], idx, val, inp["dict"], wl.L, wl.k, wl.scale, wl.c, idx.shape[1], out,
                                    kernel=kernel)
    except sr.SrError as e:
        assert e.status == -3 and kernel == MFMA
        return None
    torch.cuda.synchronize()
    return out


def check(oracle, wl, entries, idx=None, val=None, kernels=(GENERIC, MFMA)):
    """Both kernels against the oracle: the gather kernel computes in fp32 (the fp32-coefficient bound), the
    matrix-core kernel as for fp16 coefficient planes (the fp16 bound); an fp16 image adds its rounding."""
    inp = sr_synth.make_inputs(wl, DEV)
    if idx is None:
        idx, val = sr_synth.to_list(inp["coeff"], entries)
    U = oracle.bicubic(sr_synth.stored_numpy(inp["lr"]), wl.scale)
    ref = oracle.assemble_topk(U, idx.cpu().numpy(), val.cpu().numpy(), inp["dict"].cpu().numpy())
    got = None
    for kernel in kernels:
        out = run(inp, wl, idx, val, kernel)
        if out is None:
            continue
        got = out
        assert not torch.isnan(out).any(), f"kernel {kernel}: some output pixel was never written"
        bound = parity_bound(ref, "f32" if kernel == GENERIC else "f16", wl.lr_dtype == "f16")
        err = np.abs(out.float().cpu().numpy().astype(np.float64) - ref)
        assert (err <= bound).all(), f"kernel {kernel}: worst error {err.max():.3e}"
    assert got is not None
    return inp, idx, val, got


CASES = [
    # (N, C, h, w, scale, L, k, coeff dtype, image dtype, entries)
    (1, 3, 37, 64, 4, 72, 5, "f16", "f32", 8),        # the matrix-core family: several tiles, ragged rows
    (2, 3, 50, 96, 4, 72, 5, "f16", "f16", 8),        # two images, three tile columns, fp16 image
    (1, 3, 41, 66, 2, 72, 5, "f16", "f32", 5),        # scale 2, an odd number of entries (the lane halves hold 3 and 2)
    (1, 3, 29, 44, 3, 80, 5, "f16", "f32", 16),       # scale 3, the most entries and the most atoms of the small capacity
    (1, 3, 30, 40, 4, 128, 5, "f16", "f32", 7),       # 128 atoms: eight operand steps
    (1, 3, 20, 33, 4, 72, 5, "f16", "f32", 1),        # HR width 132: not whole tiles; one entry
    (1, 3, 25, 64, 4, 72, 5, "f16", "f32", 17),       # one entry too many for the matrix-core kernel: gather kernel only
    (2, 3, 21, 35, 3, 72, 5, "f16", "f32", 8),        # HR width 105: the last thread of a row holds one pixel
    (1, 1, 19, 23, 2, 40, 3, "f32", "f32", 4),
    (3, 2, 9, 70, 4, 128, 7, "f16", "f16", 16),       # 7x7, fp16 image, 280 wide: two tiles across
    (1, 16, 7, 5, 2, 17, 5, "f32", "f16", 1),         # sixteen channels, one entry
    (1, 3, 1, 1, 4, 9, 5, "f16", "f32", 9),           # a single LR pixel; as many entries as atoms
    (1, 3, 30, 130, 2, 256, 7, "f32", "f32", 3),      # the largest dictionary the table holds (53 KB of LDS)
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%dC%dh%dw%ds%dL%dk%d%s%s-T%d" % c)
def test_list_form_against_the_oracle(oracle, case):
    N, C, h, w, s, L, k, cd, io, T = case
    check(oracle, sr_synth.Workload("list", 60, N, C, h, w, s, L, k, cd, io, 0.0, 1.5), T)


def test_all_atoms_listed_is_the_dense_result(oracle):
    """Every atom of every pixel in the list (any order): the dense call's result within fp32 rounding."""
    wl = sr_synth.Workload("listall", 61, 1, 3, 20, 32, 4, 24, 5, "f16", "f32")
    inp, idx, val, got = check(oracle, wl, 24)
    dense = torch.empty_like(got)
    sr.sr_dict_assemble(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, dense)
    torch.cuda.synchronize()
    assert float((got - dense).abs().max()) <= 2e-5


def test_repeated_and_out_of_range_indices(oracle):
    wl = sr_synth.Workload("listrep", 62, 1, 3, 12, 16, 2, 10, 3, "f32", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    idx, val = sr_synth.to_list(inp["coeff"], 3)
    idx[:, 1] = idx[:, 0]                                        # the same atom twice: the gather kernel adds both
    check(oracle, wl, 3, idx, val, kernels=(GENERIC,))
    idx[:, 2] = 200                                              # not below L: unspecified values, but the call must return
    out = run(inp, wl, idx, val)
    assert torch.isfinite(out).all()
    # the matrix-core kernel: repeated and out-of-range atoms give unspecified but finite values, nothing else is touched
    wl = sr_synth.Workload("listrep", 62, 1, 3, 12, 16, 2, 20, 5, "f16", "f32")
    inp = sr_synth.make_inputs(wl, DEV)
    idx, val = sr_synth.to_list(inp["coeff"], 4)
    idx[:, 1] = idx[:, 0]
    idx[:, 3] = 250
    out = run(inp, wl, idx, val, MFMA)
    assert out is not None and torch.isfinite(out).all()


def test_4k_frame_top_8(oracle):
    """The 4K frame with each pixel's 8 largest coefficients: sampled pixels against the oracle."""
    wl = sr_synth.WORKLOADS["4k_dense"]
    inp = sr_synth.make_inputs(wl, DEV)
    idx, val = sr_synth.to_list(inp["coeff"], 8)
    del inp["coeff"]
    got = run(inp, wl, idx, val, MFMA)
    assert got is not None and not torch.isnan(got).any()
    slow = run(inp, wl, idx, val, GENERIC)
    assert float((got - slow).abs().max()) <= 2e-5
    rows = (1000, 1016)
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    ref = oracle.assemble_topk(U, idx.cpu().numpy(), val.cpu().numpy(), inp["dict"].cpu().numpy(), rows=rows)
    for y0, y1 in (rows,):
        err = np.abs(got[:, :, y0:y1].cpu().numpy().astype(np.float64) - ref[:, :, y0:y1])
        assert (err <= parity_bound(ref[:, :, y0:y1], "f16")).all(), f"worst error {err.max():.3e}"
    for band in ((0, 8), (wl.H - 8, wl.H)):
        ref = oracle.assemble_topk(U, idx.cpu().numpy(), val.cpu().numpy(), inp["dict"].cpu().numpy(), rows=band)
        err = np.abs(got[:, :, band[0]:band[1]].cpu().numpy().astype(np.float64) - ref[:, :, band[0]:band[1]])
        assert (err <= parity_bound(ref[:, :, band[0]:band[1]], "f16")).all(), f"rows {band}: worst error {err.max():.3e}"


def test_random_shapes_both_list_kernels_agree():
    """Seeded random frames and list lengths: the matrix-core form against the gather kernel (itself checked against
    the oracle above).  Both widen the same stored values; they differ by fp32 rounding order and by the 2^-22
    residue of the two-operand dictionary: 5e-5 * max(1, max|out|), plus fp16 rounding for an fp16 image."""
    rng = np.random.default_rng(20230318)
    compared = 0
    for index in range(60):
        s = int(rng.choice([2, 3, 4]))
        h, w = int(rng.integers(1, 40)), int(rng.integers(1, 50))
        if (w * s) % 4:
            w = 4 * ((w + 3) // 4)
        n = int(rng.choice([1, 1, 2]))
        L = int(rng.choice([72, 72, 40, 100, 128, 9]))
        T = int(rng.integers(1, min(16, L) + 1))
        io = str(rng.choice(["f32", "f16"]))
        wl = sr_synth.Workload("listr", 400 + index, n, 3, h, w, s, L, 5, "f16", io, 0.0, 1.5)
        inp = sr_synth.make_inputs(wl, DEV)
        idx, val = sr_synth.to_list(inp["coeff"], T)
        a = run(inp, wl, idx, val, MFMA)
        assert a is not None, f"{wl} T={T}: this case belongs to the matrix-core kernel"
        b = run(inp, wl, idx, val, GENERIC)
        assert torch.isfinite(a).all(), f"{wl}: some output pixel was never written"
        scale = max(1.0, float(b.float().abs().max()))
        tol = (5e-5 + (2.0 ** -10 if io == "f16" else 0.0)) * scale
        err = float((a.float() - b.float()).abs().max())
        assert err <= tol, f"{wl} T={T}: kernels differ by {err:.3e} > {tol:.1e}"
        compared += 1
    assert compared == 60


def test_list_tensors_at_odd_addresses(oracle):
    """The index tensor needs no alignment and the values only their own (2 bytes): both kernels must take views that
    start in the middle of a word (the matrix-core kernel reads four indices and four values at a time)."""
    wl = sr_synth.Workload("listodd", 63, 1, 3, 23, 36, 4, 72, 5, "f16", "f32", 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    idx, val = sr_synth.to_list(inp["coeff"], 6)
    ibuf = torch.zeros(idx.numel() + 8, device=DEV, dtype=torch.uint8)
    vbuf = torch.zeros(val.numel() + 8, device=DEV, dtype=val.dtype)
    for shift_i, shift_v in ((1, 1), (3, 2), (2, 3)):
        iv = ibuf[shift_i:shift_i + idx.numel()].view(idx.shape)
        vv = vbuf[shift_v:shift_v + val.numel()].view(val.shape)
        iv.copy_(idx)
        vv.copy_(val)
        assert iv.data_ptr() % 4 == shift_i % 4 and vv.data_ptr() % 8 == (2 * shift_v) % 8
        check(oracle, wl, 6, iv, vv)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_list_call_replays_inside_a_captured_graph(kernel):
    """One kernel, no allocation, and the matrix-core form clears and restores its LDS scratch itself: the call
    can be captured in a HIP graph.  Three replays with new inputs copied into the captured buffers and eager work
    in between, each compared with an eager call."""
    wl = sr_synth.Workload("listg", 64, 1, 3, 40, 64, 4, 72, 5, "f16", "f32", 0.0, 1.5)
    first = sr_synth.make_inputs(wl, DEV)
    idx0, val0 = sr_synth.to_list(first["coeff"], 8)
    lr, idx, val, D = first["lr"].clone(), idx0.clone(), val0.clone(), first["dict"].clone()
    out = torch.zeros((wl.n, wl.c, wl.H, wl.W), device=DEV)
    call = lambda: sr.sr_dict_assemble_list_ex(lr, idx, val, D, wl.L, wl.k, wl.scale, wl.c, 8, out, kernel=kernel)
    call()                                                                   # warm-up outside capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        fresh = sr_synth.make_inputs(sr_synth.scaled(wl, index=wl.index + 1 + rep), DEV)
        fi, fv = sr_synth.to_list(fresh["coeff"], 8)
        lr.copy_(fresh["lr"]); idx.copy_(fi); val.copy_(fv); D.copy_(fresh["dict"])
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager = run(fresh, wl, fi, fv, kernel)
        assert torch.equal(out, eager), f"replay {rep}"
