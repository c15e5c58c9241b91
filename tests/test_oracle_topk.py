"""Pins of the oracle's per-pixel list form (an extension beyond the paper: coefficients as T
(atom index, value) entries per pixel).  It has a plain definition - Eq. 2 restricted to the listed
terms - so it is pinned by the dense form (itself pinned) on the scattered list, and by cases whose
answer is known by hand."""
import numpy as np
import pytest


def _case(rng, n=2, c=2, H=9, W=11, L=13, k=3, T=4, dtype=np.float32):
    U = rng.random((n, c, H, W))
    D = rng.standard_normal((L, k, k))
    index = np.stack([rng.permutation(L)[:T] for _ in range(n * H * W)]).reshape(n, H, W, T).transpose(0, 3, 1, 2)
    index = np.ascontiguousarray(index.astype(np.uint8))
    value = rng.standard_normal((n, T, H, W)).astype(dtype)
    return U, index, value, D


def _scatter(index, value, L):
    n, T, H, W = index.shape
    dense = np.zeros((n, L, H, W), dtype=np.float64)
    for t in range(T):
        np.add.at(dense, (np.arange(n)[:, None, None], index[:, t], np.arange(H)[None, :, None], np.arange(W)[None, None, :]),
                  value[:, t].astype(np.float64))
    return dense


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("k,T", [(3, 1), (3, 4), (5, 8), (7, 3)])
def test_equals_the_dense_form_on_the_scattered_list(oracle, dtype, k, T):
    rng = np.random.default_rng(100 * k + T)
    U, index, value, D = _case(rng, k=k, T=T, dtype=dtype)
    got = oracle.assemble_topk(U, index, value, D)
    want = oracle.assemble(U, _scatter(index, value, D.shape[0]), D)
    assert np.abs(got - want).max() <= 1e-12 * max(1.0, np.abs(want).max())


def test_hand_made_lists(oracle):
    rng = np.random.default_rng(5)
    U = rng.random((1, 1, 6, 7))
    D = np.zeros((4, 3, 3))
    D[0, 1, 1] = 1.0          # centre: the pixel itself
    D[1, 1, 2] = 1.0          # right neighbour
    D[2, 0, 1] = 1.0          # upper neighbour
    D[3] = 1.0 / 9.0          # box filter
    index = np.zeros((1, 2, 6, 7), dtype=np.uint8)
    value = np.zeros((1, 2, 6, 7), dtype=np.float32)
    index[0, 0], value[0, 0] = 0, 2.0                 # 2 x the pixel ...
    index[0, 1], value[0, 1] = 1, -1.0                # ... minus its right neighbour (replicated at the border)
    got = oracle.assemble_topk(U, index, value, D)[0, 0]
    right = np.concatenate([U[0, 0][:, 1:], U[0, 0][:, -1:]], axis=1)
    assert np.allclose(got, 2.0 * U[0, 0] - right, atol=1e-15)
    # the same atom listed twice counts twice; a zero value contributes nothing whatever its index
    index[0, 1], value[0, 1] = 0, 0.5
    assert np.allclose(oracle.assemble_topk(U, index, value, D)[0, 0], 2.5 * U[0, 0], atol=1e-15)
    index[0, 1], value[0, 1] = 3, 0.0
    assert np.allclose(oracle.assemble_topk(U, index, value, D)[0, 0], 2.0 * U[0, 0], atol=1e-15)
    # per-pixel choice: upper neighbour on even columns, the pixel itself on odd ones
    index[0, 0, :, 0::2], index[0, 0, :, 1::2] = 2, 0
    value[0, 0], value[0, 1] = 1.0, 0.0
    up = np.concatenate([U[0, 0][:1], U[0, 0][:-1]], axis=0)
    want = U[0, 0].copy()
    want[:, 0::2] = up[:, 0::2]
    assert np.allclose(oracle.assemble_topk(U, index, value, D)[0, 0], want, atol=1e-15)


def test_linear_in_the_values_rows_and_bad_indices(oracle):
    rng = np.random.default_rng(6)
    U, index, value, D = _case(rng, T=5, k=5, L=9)
    a = oracle.assemble_topk(U, index, value, D)
    b = oracle.assemble_topk(U, index, (4.0 * value).astype(np.float32), D)       # exact in fp32
    assert np.allclose(b, 4.0 * a, rtol=1e-12, atol=1e-12)
    part = oracle.assemble_topk(U, index, value, D, rows=(2, 5))
    assert np.array_equal(part[:, :, 2:5], a[:, :, 2:5]) and not part[:, :, :2].any() and not part[:, :, 5:].any()
    index[0, 0, 0, 0] = 9                               # not below L
    with pytest.raises(ValueError):
        oracle.assemble_topk(U, index, value, D)
