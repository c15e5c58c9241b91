"""GPU parity on seeded random shapes: frame sizes, scales, atom counts, kernel sizes,
storage types, batch sizes, kept lists and tile shapes drawn at random, so that ragged
edges, partial tiles and the shares of the tile walk are hit in combinations the
hand-picked cases do not list.

  * about a hundred small cases: every kernel that takes the case against the CPU oracle,
    element by element, with the tolerances of test_gpu_parity.py;
  * a few hundred cases: the matrix-core kernel against the generic kernel (itself
    checked against the oracle above and in test_gpu_parity.py).  Both read the same
    stored values and accumulate in fp32, so they may differ by fp32 rounding order
    only: 5e-5 * max(1, max|out|), plus fp16 rounding when the output is fp16.
"""
import numpy as np
import pytest
import torch

import paper_2303_08999_amd as sr
import sr_synth
from test_gpu_parity import DEV, GENERIC, MFMA, host, planned, run_gpu, tolerance_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sr.load()


def draw(rng, index, max_h, max_w):
    k = int(rng.choice([3, 5, 5, 5, 7]))
    s = int(rng.choice([2, 3, 4]))
    C = int(rng.choice([1, 2, 3, 3, 4]))
    N = int(rng.choice([1, 1, 2, 3, 9]))
    cd = str(rng.choice(["f16", "f16", "f32", "f8", "bf16"]))
    io = str(rng.choice(["f32", "f16"]))
    L = int(rng.integers(1, 73)) if k != 7 else int(rng.choice([16, 72, 128, int(rng.integers(1, 129))]))
    h, w = int(rng.integers(1, max_h)), int(rng.integers(1, max_w))
    wl = sr_synth.Workload("random", 100 + index, N, C, h, w, s, L, k, cd, io, 0.0, 1.5)
    kept = gamma = None
    if rng.random() < 0.4:
        nk = int(rng.integers(1, L + 1))
        kept = np.sort(rng.choice(L, size=nk, replace=False)).astype(np.int32)
        if rng.random() < 0.5:
            gamma = rng.uniform(0.5, 1.5, size=nk).astype(np.float32)
    tile = int(rng.choice([0, 0, 0, 1, 2, 3, 4, 5]))
    return wl, kept, gamma, tile


def test_random_shapes_against_the_oracle(oracle):
    rng = np.random.default_rng(20230316)
    checked = {GENERIC: 0, MFMA: 0}
    for index in range(96):
        wl, kept, gamma, tile = draw(rng, index, 40, 60)
        inp = sr_synth.make_inputs(wl, DEV)
        hi = host(inp)
        ref = oracle.dict_assemble(hi["lr"], hi["coeff"], hi["dict"], wl.scale, kept=kept, gamma=gamma)
        for kernel in (GENERIC, MFMA):
            t = tile if kernel == MFMA else 0
            if planned(inp, wl, kernel, kept, t) != kernel:
                continue
            got = run_gpu(inp, wl, kernel, kept, gamma, t).float().cpu().numpy()
            assert not np.isnan(got).any(), f"{wl}: some output pixel was never written"
            worst, tol, ok = tolerance_ok(got, ref, wl.coeff_dtype, wl.lr_dtype == "f16")
            assert ok, f"{wl} kept {kept} tile {t} kernel {kernel}: worst error {worst:.3e} exceeds {tol:.0e}"
            checked[kernel] += 1
    assert checked[GENERIC] == 96 and checked[MFMA] >= 20, checked


@pytest.mark.parametrize("seed, count, max_h, max_w", [(1, 600, 70, 110), (2, 100, 300, 500)])
def test_random_shapes_kernels_agree(seed, count, max_h, max_w):
    rng = np.random.default_rng(seed)
    compared = 0
    for index in range(count):
        wl, kept, gamma, tile = draw(rng, index, max_h, max_w)
        if max_h > 100 and wl.n > 2:
            continue
        inp = sr_synth.make_inputs(wl, DEV)
        if tile != 0 and planned(inp, wl, MFMA, kept, tile) != MFMA:
            tile = 0                                    # a tile index this case does not have: its default shape
        if planned(inp, wl, MFMA, kept, tile) != MFMA:
            continue
        a = run_gpu(inp, wl, MFMA, kept, gamma, tile).float()
        b = run_gpu(inp, wl, GENERIC, kept, gamma, 0).float()
        assert torch.isfinite(a).all(), f"{wl}: some output pixel was never written"
        scale = max(1.0, float(b.abs().max()))
        tol = (5e-5 + (2.0 ** -10 if wl.lr_dtype == "f16" else 0.0)) * scale
        err = float((a - b).abs().max())
        assert err <= tol, f"{wl} kept {kept} gamma {gamma is not None} tile {tile}: kernels differ by {err:.3e} > {tol:.1e}"
        compared += 1
    assert compared >= count // 5, compared          # the others are cases the matrix-core kernel does not take
