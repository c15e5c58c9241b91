"""Pins of the oracle's move from pixel-major coefficient storage [N][H][W][L] (an extension of the storage
formats: what a channels-last producer writes) to the planar order the definition reads:
  * a hand-written example with every element different (tests/golden/pixel_major_example.txt),
  * numpy's own axis move (an independent library routine) on random tensors of every storage size,
  * the whole path: pixel-major coefficients give what their planar copy gives."""
import os

import numpy as np
import pytest


def test_hand_written_example(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "pixel_major_example.txt")
    rows = [[int(v) for v in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    stored, planar = np.array(rows[0], dtype=np.float32), np.array(rows[1], dtype=np.float32)
    got = oracle.pixel_major_to_planar(stored.reshape(1, 2, 3, 2))          # H = 2, W = 3, L = 2
    assert got.shape == (1, 2, 2, 3)
    assert np.array_equal(got.reshape(-1), planar)


@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.uint8, np.uint16])
def test_against_the_library_axis_move(oracle, dtype):
    rng = np.random.default_rng(5)
    x = rng.integers(0, 200, size=(2, 5, 7, 3)).astype(dtype)               # [N][H][W][L], no two sizes alike
    got = oracle.pixel_major_to_planar(x)
    assert got.dtype == x.dtype and np.array_equal(got, np.moveaxis(x, 3, 1))


def test_whole_path_with_pixel_major_coefficients_is_the_planar_result(oracle):
    rng = np.random.default_rng(6)
    lr = rng.random((1, 2, 4, 5)).astype(np.float32)
    D = rng.standard_normal((6, 3, 3)).astype(np.float32)
    planar = rng.standard_normal((1, 6, 8, 10)).astype(np.float32)
    pm = np.ascontiguousarray(np.moveaxis(planar, 1, 3))
    a = oracle.dict_assemble(lr, planar, D, 2)
    b = oracle.dict_assemble(lr, pm, D, 2, pixel_major=True)
    assert np.array_equal(a, b)
