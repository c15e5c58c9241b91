"""Pins of the oracle's move from the blocked coefficient storage (an extension of the storage formats: the order in
which a matrix-core kernel consumes the coefficients) to the planar order the definition reads:
  * positions worked by hand (tests/golden/blocked_example.txt): an element placed there, and only there, must arrive at
    its (atom, row, column),
  * numpy's own reshape and axis move (an independent library routine) on random tensors of every storage size, with and
    without the last 8-atom piece,
  * it is a bijection: every stored element arrives exactly once,
  * the whole path: blocked coefficients give what their planar copy gives; sizes the order does not exist for are refused."""
import os

import numpy as np
import pytest


def numpy_blocked(planar):
    """planar [N][L][H][W] -> blocked [N][H][W / 128][128 * L] with numpy's reshape / transpose."""
    n, L, H, W = planar.shape
    full, units = L // 16, W // 128
    x = planar.reshape(n, L, H, units, 32, 4)
    parts = []
    if full:
        parts.append(x[:, :16 * full].reshape(n, full, 2, 8, H, units, 32, 4).transpose(0, 4, 5, 7, 1, 2, 6, 3).reshape(n, H, units, 4, -1))
    if L % 16:
        parts.append(x[:, 16 * full:].reshape(n, 2, 4, H, units, 32, 4).transpose(0, 3, 4, 6, 1, 5, 2).reshape(n, H, units, 4, -1))
    return np.ascontiguousarray(np.concatenate(parts, axis=-1).reshape(n, H, units, 128 * L))


def test_hand_worked_positions(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "blocked_example.txt")
    rows = [[int(v) for v in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    L, H, W = 24, 2, 256
    for l, y, x, index in rows:
        stored = np.zeros((1, H, W // 128, 128 * L), dtype=np.float32)
        stored.reshape(-1)[index] = 7.0
        got = oracle.blocked_to_planar(stored)
        assert got.shape == (1, L, H, W)
        assert got[0, l, y, x] == 7.0 and np.count_nonzero(got) == 1, (l, y, x, index)


@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.uint8, np.uint16])
@pytest.mark.parametrize("L", [8, 16, 24, 72])
def test_against_the_library_axis_moves(oracle, dtype, L):
    rng = np.random.default_rng(L)
    planar = rng.integers(0, 250, size=(2, L, 3, 256)).astype(dtype)
    got = oracle.blocked_to_planar(numpy_blocked(planar))
    assert got.dtype == planar.dtype and np.array_equal(got, planar)


def test_every_stored_element_arrives_once(oracle):
    L, H, W = 40, 2, 128
    stored = np.arange(H * W * L, dtype=np.float64).reshape(1, H, W // 128, 128 * L)
    got = oracle.blocked_to_planar(stored)
    assert np.array_equal(np.sort(got.reshape(-1)), stored.reshape(-1))
    # a slot is 32 pixels x L atoms: the elements of the first slot are the pixels 0, 4, 8, ... of the first unit
    first_slot = got[0, :, 0, 0:128:4]
    assert first_slot.min() == 0 and first_slot.max() == 32 * L - 1


def test_whole_path_and_refusals(oracle):
    rng = np.random.default_rng(9)
    lr = rng.random((1, 2, 3, 64)).astype(np.float32)                       # x2 -> 6 x 128
    D = rng.standard_normal((24, 3, 3)).astype(np.float32)
    planar = rng.standard_normal((1, 24, 6, 128)).astype(np.float32)
    a = oracle.dict_assemble(lr, planar, D, 2)
    b = oracle.dict_assemble(lr, numpy_blocked(planar), D, 2, blocked=True)
    assert np.array_equal(a, b)
    with pytest.raises(ValueError):
        oracle.blocked_to_planar(np.zeros((1, 2, 1, 100 * 24), dtype=np.float32))       # not whole units of 128 pixels
    with pytest.raises(ValueError):
        oracle.blocked_to_planar(np.zeros((1, 2, 1, 128 * 12), dtype=np.float32))       # L = 12: not whole groups of 8


def test_generator_writes_the_same_order():
    import torch
    import sr_synth
    rng = np.random.default_rng(10)
    for L in (8, 24, 72):
        planar = rng.integers(0, 250, size=(2, L, 3, 256)).astype(np.float32)
        assert np.array_equal(sr_synth.to_blocked(torch.from_numpy(planar)).numpy(), numpy_blocked(planar))
