"""Pins of the oracle's pixel-shuffle (paper section II-B, stage 2: the coefficient network ends
in a pixel-shuffle layer).  The paper prints no example; the operation is fixed by the layer's
published definition, out[l][y*s+i][x*s+j] = in[l*s*s + i*s + j][y][x]:
  * a hand-written 2x2 case (tests/golden/pixel_shuffle_example.txt),
  * torch's pixel_shuffle on the CPU (an independent library routine),
  * the index identity itself on random shapes, every scale, every storage width,
  * the inverse library routine (pixel_unshuffle) brings the input back."""
import os

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_hand_written_example(oracle):
    rows = [l.split("#")[0].split() for l in open(os.path.join(ROOT, "tests", "golden", "pixel_shuffle_example.txt"))]
    rows = [[int(v) for v in r] for r in rows if r]
    n_in = 8                                         # 8 channels of 1 x 2 (two atoms at scale 2)
    x = np.array(rows[:n_in], dtype=np.float32).reshape(1, 8, 1, 2)
    want = np.array(rows[n_in:], dtype=np.float32).reshape(1, 2, 2, 4)
    assert np.array_equal(oracle.pixel_shuffle(x, 2), want)


@pytest.mark.parametrize("scale", [2, 3, 4])
@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.uint8, np.uint16, np.float64])
def test_against_the_library_routine_and_the_index_identity(oracle, scale, dtype):
    rng = np.random.default_rng(scale * 10 + np.dtype(dtype).itemsize)
    n, L, h, w = 2, 5, 3, 7
    x = rng.integers(0, 250, size=(n, L * scale * scale, h, w)).astype(dtype)
    got = oracle.pixel_shuffle(x, scale)
    assert got.dtype == x.dtype and got.shape == (n, L, h * scale, w * scale)
    lib = torch.nn.functional.pixel_shuffle(torch.from_numpy(x.astype(np.float64)), scale).numpy()
    assert np.array_equal(got.astype(np.float64), lib)
    for _ in range(200):
        b, l, y, xx, i, j = (int(rng.integers(0, m)) for m in (n, L, h, w, scale, scale))
        assert got[b, l, y * scale + i, xx * scale + j] == x[b, l * scale * scale + i * scale + j, y, xx]
    back = torch.nn.functional.pixel_unshuffle(torch.from_numpy(got.astype(np.float64)), scale).numpy()
    assert np.array_equal(back, x.astype(np.float64))


def test_whole_path_with_pre_shuffle_coefficients_is_the_planar_result(oracle):
    rng = np.random.default_rng(3)
    s, L, k = 3, 4, 3
    lr = rng.random((1, 2, 4, 5))
    pre = rng.random((1, L * s * s, 4, 5)).astype(np.float32)
    D = rng.standard_normal((L, k, k))
    planar = torch.nn.functional.pixel_shuffle(torch.from_numpy(pre), s).numpy()
    assert np.array_equal(oracle.dict_assemble(lr, pre, D, s, pre_shuffle=True), oracle.dict_assemble(lr, planar, D, s))
    # a transposed sub-pixel order (j major instead of i major) must change the result
    wrong = pre.reshape(1, L, s, s, 4, 5).transpose(0, 1, 3, 2, 4, 5).reshape(pre.shape)
    assert not np.array_equal(oracle.dict_assemble(lr, np.ascontiguousarray(wrong), D, s, pre_shuffle=True),
                              oracle.dict_assemble(lr, planar, D, s))
