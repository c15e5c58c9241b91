"""The entry point that allocates nothing (sr_atom_gram_static, for callers that cannot call
hipMalloc or pass a workspace) against the existing one (sr_atom_gram, caller's workspace):
same kernels, same summation order, so the normal equations must be identical.  Two calls in a
row on the library's built-in scratch, the second on a smaller input, so that whatever the
first call left in the buffer would show."""
import ctypes

import pytest

torch = pytest.importorskip("torch")
import paper_2303_08999_amd as sr
import sr_synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _problem(N, C, h, w, s, L, k, cd, seed):
    wl = sr_synth.Workload("noalloc", seed, N, C, h, w, s, L, k, cd, "f32", 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    up = torch.empty((N, C, wl.H, wl.W), device=DEV)
    sr.sr_bicubic_upsample(inp["lr"], s, C, up)
    g = torch.Generator(device=DEV).manual_seed(900 + seed)
    target = torch.rand((N, C, wl.H, wl.W), device=DEV, generator=g)
    return wl, inp, up, target


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    big = _problem(1, 3, 64, 80, 4, 72, 5, "f16", 41)        # 1280 runs: every workgroup writes partial sums
    small = _problem(2, 1, 9, 11, 2, 20, 3, "f32", 42)       # fewer atoms, fewer blocks, most workgroups idle
    results = []
    for wl, inp, up, target in (big, small):
        want = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, 1)
        got = torch.full((wl.L * wl.L + wl.L + 2,), float("nan"), device=DEV, dtype=torch.float64)
        sr.sr_atom_gram_static(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, 1, got)
        results.append((want, got))
    torch.cuda.synchronize()
    for (want, got), name in zip(results, ("first call", "second, smaller call")):
        assert bool(torch.isfinite(got).all()), name
        assert torch.equal(want, got), name
    # once more in the other order, with a lattice stride: the buffer now holds the small problem's sums
    for (wl, inp, up, target), stride in ((big, 3), (small, 2)):
        want = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, stride)
        got = torch.empty_like(want)
        sr.sr_atom_gram_static(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, stride, got)
        torch.cuda.synchronize()
        assert torch.equal(want, got)


def test_static_scratch_entry_point_refuses_what_its_buffer_cannot_hold():
    wl, inp, up, target = _problem(1, 1, 8, 8, 2, 80, 3, "f32", 43)
    normal = torch.zeros(wl.L * wl.L + wl.L + 2, device=DEV, dtype=torch.float64)
    with pytest.raises(sr.SrError) as err:
        sr.sr_atom_gram_static(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, 1, normal)
    assert err.value.status == -8 and "scratch" in str(err.value)
    torch.cuda.synchronize()
    assert float(normal.abs().sum()) == 0.0                     # nothing was launched
    # 79 atoms (five column blocks) is the most it holds
    wl, inp, up, target = _problem(1, 1, 8, 8, 2, 79, 3, "f32", 44)
    want = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, 1)
    got = torch.empty_like(want)
    sr.sr_atom_gram_static(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, 1, got)
    torch.cuda.synchronize()
    assert torch.equal(want, got)
