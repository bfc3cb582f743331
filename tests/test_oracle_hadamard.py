"""Pins for the oracle's Hadamard transform (paper, Methodology: Sylvester form,
block-diagonal H, orthogonality, products need no inverse transform)."""
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import capi, definitional


def test_h2_matches_hand_written_matrix(golden_dir):
    H2 = np.loadtxt(os.path.join(golden_dir, "hadamard_h2.txt"), dtype=np.int64)
    assert np.array_equal(capi.hadamard_matrix(2).astype(np.int64), H2)
    assert np.array_equal(definitional.hadamard(4), H2)


@pytest.mark.parametrize("k", range(0, 9))
def test_orthogonal_symmetric_and_textbook(k):
    n = 1 << k
    H = capi.hadamard_matrix(k).astype(np.int64)
    assert set(np.unique(H)) <= {-1, 1}
    assert np.array_equal(H, H.T)                               # symmetric
    assert np.array_equal(H @ H.T, n * np.eye(n, dtype=np.int64))  # H H^T = n I
    assert np.array_equal(H, scipy.linalg.hadamard(n).astype(np.int64))  # library routine
    assert np.array_equal(H, definitional.hadamard(n))          # popcount closed form


@pytest.mark.parametrize("D,n,expect", [(576, 64, 64), (1152, 64, 64), (320, 32, 32),
                                        (320, 64, 64), (27, 64, 1), (100, 64, 4), (128, 16, 16),
                                        (561, 32, 1), (405, 8, 1), (96, 64, 32), (4096, 256, 256)])
def test_block_order_is_largest_dividing_power_of_two(D, n, expect):
    assert capi.n_eff(D, n) == expect
    assert definitional.n_eff(D, n) == expect
    assert D % expect == 0 and expect <= n


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("n", [1, 2, 4, 16, 64, 256])
def test_integer_inputs_equal_exact_matrix_product(axis, n):
    # integer-valued inputs small enough that every partial sum is exact in
    # binary32: any summation order gives the same answer, so this pins values
    rng = np.random.default_rng(100 + n + axis)
    shape = (3, 2 * n) if axis == 1 else (2 * n, 3)
    T = rng.integers(-1000, 1000, size=shape).astype(np.float32)
    Y = capi.hadamard_transform(T, axis, n)
    H = scipy.linalg.hadamard(n).astype(np.int64) if n > 1 else np.ones((1, 1), dtype=np.int64)
    Ti = T.astype(np.int64)
    if axis == 1:
        want = np.concatenate([Ti[:, b * n:(b + 1) * n] @ H for b in range(2)], axis=1)
    else:
        want = np.concatenate([H @ Ti[b * n:(b + 1) * n, :] for b in range(2)], axis=0)
    assert np.array_equal(Y.astype(np.int64), want)
    assert np.all(Y == np.round(Y))


@pytest.mark.parametrize("n", [2, 8, 64, 512])
def test_round_trip_gives_n_times_input(n):
    rng = np.random.default_rng(n)
    T = rng.integers(-100, 100, size=(4, n)).astype(np.float32)
    back = capi.hadamard_transform(capi.hadamard_transform(T, 1, n), 1, n)
    assert np.array_equal(back, n * T)


def test_pairwise_tree_hand_case():
    # binary32: 1e8 + 1 == 1e8.  Tree ((1e8 + 1) + (-1e8 + 1)) = 1e8 + (-1e8) = 0,
    # while left-to-right (((1e8 + 1) - 1e8) + 1) = 1.  Row 0 of H_2 is all ones.
    x = np.array([[1e8, 1.0, -1e8, 1.0]], dtype=np.float32)
    Y = capi.hadamard_transform(x, 1, 4)
    assert Y[0, 0] == 0.0
    # row 1 (+,-,+,-): (1e8 - 1) + (-1e8 - 1) = 1e8 + -1e8 = 0
    assert Y[0, 1] == 0.0
    # row 2 (+,+,-,-): (1e8 + 1) + (1e8 - 1) = 2e8
    assert Y[0, 2] == np.float32(2e8)


def _butterfly(x, strides):
    x = x.astype(np.float32).copy()
    n = x.shape[0]
    for h in strides:
        y = x.copy()
        for p in range(n):
            if p & h:
                y[p] = np.float32(x[p ^ h] - x[p])
            else:
                y[p] = np.float32(x[p] + x[p ^ h])
        x = y
    return x


@pytest.mark.parametrize("n", [4, 16, 64, 256])
def test_tree_equals_butterfly_with_increasing_strides(n):
    # the radix-2 butterfly run with strides 1, 2, 4, ... realises the same tree
    rng = np.random.default_rng(n + 7)
    x = (rng.standard_normal(n) * 10.0 ** rng.integers(-3, 4, size=n)).astype(np.float32)
    Y = capi.hadamard_transform(x[None, :], 1, n)[0]
    strides = [1 << i for i in range(n.bit_length() - 1)]
    assert np.array_equal(Y, _butterfly(x, strides))
    assert np.array_equal(definitional.transform_line(x, n), Y)


def test_stride_order_matters_for_rounding():
    # decreasing strides compute the same values in exact arithmetic but round
    # differently somewhere: the order is part of the definition
    rng = np.random.default_rng(3)
    differs = False
    for _ in range(20):
        x = (rng.standard_normal(64) * 10.0 ** rng.integers(-3, 4, size=64)).astype(np.float32)
        Y = capi.hadamard_transform(x[None, :], 1, 64)[0]
        differs |= not np.array_equal(Y, _butterfly(x, [32, 16, 8, 4, 2, 1]))
    assert differs


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("n", [8, 64, 256])
def test_binary32_tree_close_to_binary64(axis, n):
    rng = np.random.default_rng(5 * n + axis)
    shape = (5, n) if axis == 1 else (n, 5)
    T = rng.standard_normal(shape).astype(np.float32)
    Y32 = capi.hadamard_transform(T, axis, n).astype(np.float64)
    Y64 = capi.hadamard_transform_f64(T, axis, n)
    H = scipy.linalg.hadamard(n).astype(np.float64)
    want = T.astype(np.float64) @ H if axis == 1 else H @ T.astype(np.float64)
    assert np.allclose(Y64, want, rtol=0, atol=1e-9)
    # each of the log2(n) levels adds at most 2^-24 relative error on sum |x|
    bound = np.log2(n) * 2.0 ** -24 * np.abs(T.astype(np.float64)).sum(axis=axis, keepdims=True)
    assert np.all(np.abs(Y32 - Y64) <= bound + 1e-30)


def test_products_need_no_inverse_transform():
    # (X H)(H^T W) / n == X W exactly on small integers (all three orientations
    # contract along the transformed axis)
    rng = np.random.default_rng(11)
    M, K, N, n = 6, 32, 5, 16
    X = rng.integers(-5, 6, size=(M, K)).astype(np.float32)
    W = rng.integers(-5, 6, size=(K, N)).astype(np.float32)
    XH = capi.hadamard_transform(X, 1, n).astype(np.int64)
    HW = capi.hadamard_transform(W, 0, n).astype(np.int64)
    assert np.array_equal(XH @ HW, n * (X.astype(np.int64) @ W.astype(np.int64)))
