"""GPU parity of the selection's normal equations (sr_atom_gram) against the numpy
oracle, and the whole chain on a planted problem: up-sample, normal equations, Alg. 1,
selective assembly with the kept list and gamma it returned."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2303_08999_amd as sr
import sr_synth
from oracle import select_oracle as so

pytestmark = pytest.mark.gpu
DEV = "cuda"

CASES = [
    # (N, C, h, w, scale, L, k, coeff dtype, stride)
    (1, 3, 9, 11, 2, 5, 3, "f32", 1),
    (2, 3, 12, 17, 4, 72, 5, "f16", 1),      # 3264 lattice pixels: 51 runs of 64 samples
    (1, 1, 16, 16, 3, 128, 7, "f16", 2),     # the largest atom count: 9 column blocks, 12 blocks per wavefront
    (3, 2, 10, 13, 2, 17, 7, "f32", 3),      # ragged lattice, L + 1 not a multiple of 4
    (1, 3, 40, 48, 4, 72, 5, "f16", 5),
    (1, 16, 6, 7, 2, 3, 3, "f32", 1),        # 16 channels
    (2, 3, 11, 14, 4, 40, 5, "f8", 2),       # coefficients stored as 8-bit E4M3
    (1, 3, 40, 50, 4, 72, 5, "bf16", 1),     # ... as bfloat16, several runs per workgroup
    # more runs than workgroups, so that every workgroup walks several runs and channels
    (1, 3, 64, 80, 4, 72, 5, "f16", 1),      # 1280 runs of one lattice row segment each
    (1, 1, 96, 100, 4, 20, 5, "f32", 1),     # one channel: a new run every iteration, 2688 runs
    (2, 2, 120, 130, 3, 72, 3, "f8", 2),     # two channels, two images, ragged last segment
    (1, 3, 30, 500, 2, 100, 7, "f16", 4),    # 7 x 7, 9 column blocks, stride 4: long staged segments
]


def _inputs(case):
    N, C, h, w, s, L, k, cd, stride = case
    wl = sr_synth.Workload("gram", 30, N, C, h, w, s, L, k, cd, "f32", 0.0, 1.5)
    inp = sr_synth.make_inputs(wl, DEV)
    up = torch.empty((N, C, wl.H, wl.W), device=DEV)
    sr.sr_bicubic_upsample(inp["lr"], s, C, up)
    g = torch.Generator(device=DEV).manual_seed(77 + L)
    target = torch.rand((N, C, wl.H, wl.W), device=DEV, generator=g)
    return wl, inp, up, target


@pytest.mark.parametrize("case", CASES, ids=lambda c: "N%dC%dh%dw%ds%dL%dk%d%sst%d" % c)
def test_normal_equations_match_the_oracle(oracle, case):
    wl, inp, up, target = _inputs(case)
    stride = case[-1]
    normal = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, stride)
    again = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, stride)
    torch.cuda.synchronize()
    assert torch.equal(normal, again), "the sums must not depend on the run"
    got = normal.cpu().numpy()
    L = wl.L
    G, b, hh, M = got[:L * L].reshape(L, L), got[L * L:L * L + L], got[L * L + L], got[L * L + L + 1]
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    G0, b0, hh0, M0 = so.normal_equations(U, sr_synth.stored_numpy(inp["coeff"]), inp["dict"].cpu().numpy(),
                                          target.cpu().numpy(), stride)
    assert M == M0
    assert np.array_equal(G, G.T)
    # fp32 responses (relative 1e-6 each), fp32 sums over 64 samples, double beyond
    scale = np.sqrt(np.outer(np.diag(G0), np.diag(G0)))
    assert np.abs(G - G0).max() <= 2e-5 * scale.max() and (np.abs(G - G0) <= 2e-5 * scale + 1e-12).all()
    assert (np.abs(b - b0) <= 2e-5 * np.sqrt(np.diag(G0) * hh0) + 1e-12).all()
    assert abs(hh - hh0) <= 1e-6 * hh0


def test_normal_equations_on_random_shapes(oracle):
    """Sixty seeded shapes over both kernel forms: every stride from 1 to 7, one to sixteen
    channels, all four coefficient types, atom counts around every block boundary."""
    rng = np.random.default_rng(5)
    done = 0
    while done < 60:
        k = int(rng.choice([3, 5, 5, 7]))
        s = int(rng.choice([2, 3, 4]))
        C = int(rng.choice([1, 1, 2, 3, 3, 4, 7, 16]))
        N = int(rng.choice([1, 1, 2, 3]))
        cd = str(rng.choice(["f16", "bf16", "f32", "f8"]))
        L = int(rng.choice([int(rng.integers(1, 129)), 72, 16, 31, 32, 33, 79, 80, 81, 128]))
        stride = int(rng.choice([1, 1, 2, 3, 4, 5, 7]))
        h, w = int(rng.integers(2, 60)), int(rng.integers(2, 120))
        if L * C * h * w * s * s * N > 40e6:
            continue
        done += 1
        wl = sr_synth.Workload("gramr", 300 + done, N, C, h, w, s, L, k, cd, "f32", 0.0, 1.5)
        inp = sr_synth.make_inputs(wl, DEV)
        up = torch.empty((N, C, wl.H, wl.W), device=DEV)
        sr.sr_bicubic_upsample(inp["lr"], s, C, up)
        g = torch.Generator(device=DEV).manual_seed(77 + done)
        target = torch.rand((N, C, wl.H, wl.W), device=DEV, generator=g)
        got = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, L, k, C, stride).cpu().numpy()
        G, b, hh, M = got[:L * L].reshape(L, L), got[L * L:L * L + L], got[L * L + L], got[L * L + L + 1]
        G0, b0, hh0, M0 = so.normal_equations(up.cpu().numpy().astype(np.float64), sr_synth.stored_numpy(inp["coeff"]),
                                              inp["dict"].cpu().numpy(), target.cpu().numpy(), stride)
        case = (N, C, h, w, s, L, k, cd, stride)
        scale = np.sqrt(np.outer(np.diag(G0), np.diag(G0)))
        assert M == M0 and np.array_equal(G, G.T), case
        assert np.abs(G - G0).max() <= 2e-5 * scale.max() and (np.abs(G - G0) <= 2e-5 * scale + 1e-12).all(), case
        assert (np.abs(b - b0) <= 2e-5 * np.sqrt(np.diag(G0) * hh0) + 1e-12).all(), case
        assert abs(hh - hh0) <= 1e-6 * hh0, case


def test_empty_batch_and_undersized_scratch():
    wl, inp, up, target = _inputs(CASES[0])
    z = torch.empty((0, 3, wl.H, wl.W), device=DEV)
    zc = torch.empty((0, wl.L, wl.H, wl.W), device=DEV)
    normal = sr.sr_atom_gram(z, zc, inp["dict"], z.clone(), wl.L, wl.k, 3)
    torch.cuda.synchronize()
    assert not normal.cpu().numpy().any()
    small = torch.empty(1024, device=DEV, dtype=torch.uint8)
    with pytest.raises(sr.SrError) as err:
        sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, 3, workspace=small)
    assert err.value.status == -2


def test_whole_chain_recovers_a_planted_selection(oracle):
    """The target is what the path itself produces from 6 of 40 atoms with known scales;
    the selection must find exactly them, and assembling with what it returns must
    reproduce the target."""
    wl = sr_synth.Workload("plant", 31, 2, 3, 20, 26, 4, 40, 5, "f16", "f32", 0.0, 1.0)
    inp = sr_synth.make_inputs(wl, DEV)
    planted = np.array([4, 9, 17, 22, 30, 39], dtype=np.int32)
    scales = np.array([1.5, 0.5, -1.0, 2.0, 0.75, 1.25], dtype=np.float32)
    target = torch.empty((wl.n, wl.c, wl.H, wl.W), device=DEV)
    sr.sr_dict_assemble_selective(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, target,
                                  kept=planted, gamma=scales)
    up = torch.empty_like(target)
    sr.sr_bicubic_upsample(inp["lr"], wl.scale, wl.c, up)
    normal = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], target, wl.L, wl.k, wl.c, stride=2)
    torch.cuda.synchronize()
    kept, gamma, lam = sr.sr_select_atoms(normal.cpu().numpy(), wl.L, alpha=6 / 40, delta_alpha=0.3)
    assert np.array_equal(kept, planted)
    assert np.allclose(gamma, scales, atol=2e-3)
    out = torch.empty_like(target)
    sr.sr_dict_assemble_selective(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, out,
                                  kept=kept, gamma=gamma)
    torch.cuda.synchronize()
    assert float((out - target).abs().max()) <= 5e-3
    # the oracle's selection from the oracle's normal equations agrees
    U = oracle.bicubic(inp["lr"].cpu().numpy(), wl.scale)
    G0, b0, hh0, M0 = so.normal_equations(U, inp["coeff"].cpu().numpy(), inp["dict"].cpu().numpy(),
                                          target.cpu().numpy(), 2)
    k0, g0, _ = so.select_atoms(G0, b0, hh0, M0, 6 / 40, 0.3)
    assert np.array_equal(k0, kept) and np.allclose(g0, gamma, atol=2e-3)


def test_selection_finds_the_dominant_atoms_of_the_selective_workload():
    """The selective workload gives 8 seeded atoms most of the coefficient mass.  Asked for
    8 of 72 atoms to reproduce the DENSE result, Alg. 1 must pick exactly those 8 (the
    list the workload itself derives from the mean coefficients), and assembling with its
    kept list and gamma must come closer to the dense result than the unscaled kept list."""
    wl = sr_synth.scaled(sr_synth.WORKLOADS["4k_selective"], h=90, w=120)
    inp = sr_synth.make_inputs(wl, DEV)
    shape = (wl.n, wl.c, wl.H, wl.W)
    dense, up = torch.empty(shape, device=DEV), torch.empty(shape, device=DEV)
    sr.sr_dict_assemble(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, dense)
    sr.sr_bicubic_upsample(inp["lr"], wl.scale, wl.c, up)
    normal = sr.sr_atom_gram(up, inp["coeff"], inp["dict"], dense, wl.L, wl.k, wl.c, stride=3)
    torch.cuda.synchronize()
    kept, gamma, _ = sr.sr_select_atoms(normal.cpu().numpy(), wl.L, alpha=8 / 72, delta_alpha=0.2)
    assert np.array_equal(kept, inp["kept"])
    assert np.array_equal(np.sort(sr_synth.dominant_atoms(wl)), kept)
    assert np.all(gamma > 1.0) and np.all(gamma < 1.5)          # they make up for the dropped ~13 % of the mass
    plain, scaled = torch.empty(shape, device=DEV), torch.empty(shape, device=DEV)
    sr.sr_dict_assemble_selective(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, plain, kept=kept)
    sr.sr_dict_assemble_selective(inp["lr"], inp["coeff"], inp["dict"], wl.L, wl.k, wl.scale, wl.c, scaled,
                                  kept=kept, gamma=gamma)
    torch.cuda.synchronize()
    err_plain = float(((plain - dense) ** 2).mean())
    err_scaled = float(((scaled - dense) ** 2).mean())
    assert err_scaled < 0.25 * err_plain
