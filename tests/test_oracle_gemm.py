"""Pins for the oracle's three products (CPU only).

Section 3.1 eq. (1)-(3) of arxiv 2411.01238 against: a hand-worked example, a
library float64 matmul in the unmasked case, the mask applied by a different
route (np.repeat) followed by the library matmul, central finite differences
of the forward, the adjoint identity of the bilinear form, exact zeros where
everything is dropped, and block linearity.  Shapes are never square so that a
transposed operand or a swapped block index fails.
"""
import os

import numpy as np
import pytest

from oracle import sdrop_oracle as orc

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _expand(keep, BM, BK):
    return np.repeat(np.repeat(keep.astype(np.float64), BM, axis=0), BK, axis=1)


def _case(seed=0, MB=3, KB=5, BM=4, BK=2, N=7, p=0.4):
    M, K = MB * BM, KB * BK
    X = _rand((M, K), seed)
    W = _rand((K, N), seed + 1)
    dY = _rand((M, N), seed + 2)
    keep = orc.mask(MB, KB, p, seed, 0)
    assert 0 < keep.sum() < keep.size
    return X, W, dY, keep, BM, BK, p


def test_hand_worked_example():
    v = {}
    with open(os.path.join(GOLD, "hand_2x2.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            k, *rest = line.split()
            v[k] = np.array([float(x) for x in rest]).reshape(2, 2)
    keep = v["keep"].astype(np.uint8)
    assert np.array_equal(orc.fwd(v["X"], v["W"], keep, 1, 1, 0.5), v["Y"])
    assert np.array_equal(orc.bwd_dx(v["dY"], v["W"], keep, 1, 1, 0.5), v["dX"])
    assert np.array_equal(orc.bwd_dw(v["X"], v["dY"], keep, 1, 1, 0.5), v["dW"])


def test_block_orientation_rows_are_BM_columns_are_BK():
    # X is 4x2 with BM=2, BK=1: the keep grid is 2x2 and keep[1,0]=0 zeroes
    # rows 2-3 of column 0 only
    X = np.arange(1.0, 9.0).reshape(4, 2)
    W = np.eye(2)
    keep = np.array([[1, 1], [0, 1]], dtype=np.uint8)
    Y = orc.fwd(X, W, keep, 2, 1, 0.0)
    want = X.copy()
    want[2:4, 0] = 0.0
    assert np.array_equal(Y, want)


def test_unmasked_equals_library_matmul():
    X, W, dY, keep, BM, BK, _ = _case(seed=3)
    ones = np.ones_like(keep)
    np.testing.assert_allclose(orc.fwd(X, W, ones, BM, BK, 0.0), X @ W, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.bwd_dx(dY, W, ones, BM, BK, 0.0), dY @ W.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.bwd_dw(X, dY, ones, BM, BK, 0.0), X.T @ dY, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("p", [0.1, 0.5, 0.7])
def test_mask_then_dense_equals_oracle(p):
    X, W, dY, keep, BM, BK, _ = _case(seed=5, p=p)
    m = _expand(keep, BM, BK)
    s = 1.0 / (1.0 - p)
    np.testing.assert_allclose(orc.fwd(X, W, keep, BM, BK, p), s * ((X * m) @ W), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.bwd_dx(dY, W, keep, BM, BK, p), s * ((dY @ W.T) * m), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.bwd_dw(X, dY, keep, BM, BK, p), s * ((X * m).T @ dY), rtol=1e-12, atol=1e-12)


def test_scale_is_one_over_one_minus_p():
    X, W, dY, keep, BM, BK, _ = _case(seed=6)
    for p in (0.25, 0.5):
        np.testing.assert_allclose(orc.fwd(X, W, keep, BM, BK, p),
                                   orc.fwd(X, W, keep, BM, BK, 0.0) / (1 - p), rtol=1e-13)
        np.testing.assert_allclose(orc.bwd_dx(dY, W, keep, BM, BK, p),
                                   orc.bwd_dx(dY, W, keep, BM, BK, 0.0) / (1 - p), rtol=1e-13)
        np.testing.assert_allclose(orc.bwd_dw(X, dY, keep, BM, BK, p),
                                   orc.bwd_dw(X, dY, keep, BM, BK, 0.0) / (1 - p), rtol=1e-13)


def test_all_dropped_gives_exact_zeros():
    X, W, dY, keep, BM, BK, _ = _case(seed=7)
    none = np.zeros_like(keep)
    for p in (0.5, 1.0):
        for out in (orc.fwd(X, W, none, BM, BK, p), orc.bwd_dx(dY, W, none, BM, BK, p),
                    orc.bwd_dw(X, dY, none, BM, BK, p)):
            assert np.all(out == 0.0) and not np.any(np.signbit(out))


def test_dx_is_exactly_zero_on_dropped_blocks_only():
    X, W, dY, keep, BM, BK, p = _case(seed=8)
    dX = orc.bwd_dx(dY, W, keep, BM, BK, p)
    m = _expand(keep, BM, BK).astype(bool)
    assert np.all(dX[~m] == 0.0) and not np.any(np.signbit(dX[~m]))
    assert np.all(dX[m] != 0.0)


def test_block_linearity_of_forward():
    X, W, dY, keep, BM, BK, p = _case(seed=9)
    total = np.zeros((X.shape[0], W.shape[1]))
    for i, j in zip(*np.nonzero(keep)):
        one = np.zeros_like(keep)
        one[i, j] = 1
        total += orc.fwd(X, W, one, BM, BK, p)
    np.testing.assert_allclose(total, orc.fwd(X, W, keep, BM, BK, p), rtol=1e-12, atol=1e-12)


def test_dropped_blocks_are_selected_not_multiplied():
    X, W, dY, keep, BM, BK, p = _case(seed=10)
    m = _expand(keep, BM, BK).astype(bool)
    Xp = X.copy()
    Xp[~m] = np.nan
    assert np.array_equal(orc.fwd(Xp, W, keep, BM, BK, p), orc.fwd(X, W, keep, BM, BK, p))
    assert np.array_equal(orc.bwd_dw(Xp, dY, keep, BM, BK, p), orc.bwd_dw(X, dY, keep, BM, BK, p))


def test_gradients_match_central_differences():
    X, W, dY, keep, BM, BK, p = _case(seed=11)

    def loss(Xa, Wa):
        return float(np.sum(orc.fwd(Xa, Wa, keep, BM, BK, p) * dY))

    dX = orc.bwd_dx(dY, W, keep, BM, BK, p)
    dW = orc.bwd_dw(X, dY, keep, BM, BK, p)
    h = 1e-3
    for t in range(4):
        E = _rand(X.shape, 100 + t)
        fd = (loss(X + h * E, W) - loss(X - h * E, W)) / (2 * h)
        assert abs(fd - np.sum(dX * E)) <= 1e-8 * max(1.0, abs(fd))
        F = _rand(W.shape, 200 + t)
        fd = (loss(X, W + h * F) - loss(X, W - h * F)) / (2 * h)
        assert abs(fd - np.sum(dW * F)) <= 1e-8 * max(1.0, abs(fd))
    # single-coordinate directions catch an index slip that a random direction averages out
    for (r, c) in ((0, 0), (5, 3), (X.shape[0] - 1, X.shape[1] - 1)):
        E = np.zeros_like(X)
        E[r, c] = 1.0
        fd = (loss(X + h * E, W) - loss(X - h * E, W)) / (2 * h)
        assert abs(fd - dX[r, c]) <= 1e-8 * max(1.0, abs(fd))
    for (r, c) in ((0, 0), (4, 6), (W.shape[0] - 1, W.shape[1] - 1)):
        F = np.zeros_like(W)
        F[r, c] = 1.0
        fd = (loss(X, W + h * F) - loss(X, W - h * F)) / (2 * h)
        assert abs(fd - dW[r, c]) <= 1e-8 * max(1.0, abs(fd))


def test_adjoint_identity():
    X, W, dY, keep, BM, BK, p = _case(seed=12)
    a = np.sum(dY * orc.fwd(X, W, keep, BM, BK, p))
    b = np.sum(orc.bwd_dx(dY, W, keep, BM, BK, p) * X)
    c = np.sum(orc.bwd_dw(X, dY, keep, BM, BK, p) * W)
    assert abs(a - b) <= 1e-10 * abs(a) and abs(a - c) <= 1e-10 * abs(a)


def test_single_entry_functions_equal_whole_products():
    X, W, dY, keep, BM, BK, p = _case(seed=13, MB=4, KB=6, BM=8, BK=4, N=10)
    rng = np.random.default_rng(0)
    M, K = X.shape
    N = W.shape[1]
    Y = orc.fwd(X, W, keep, BM, BK, p)
    dX = orc.bwd_dx(dY, W, keep, BM, BK, p)
    dW = orc.bwd_dw(X, dY, keep, BM, BK, p)
    r, c = rng.integers(0, M, 50), rng.integers(0, N, 50)
    np.testing.assert_allclose(orc.fwd_at(X, W, keep, BM, BK, p, r, c), Y[r, c], rtol=1e-13, atol=1e-13)
    r, c = rng.integers(0, M, 50), rng.integers(0, K, 50)
    np.testing.assert_allclose(orc.bwd_dx_at(dY, W, keep, BM, BK, p, r, c), dX[r, c], rtol=1e-13, atol=1e-13)
    r, c = rng.integers(0, K, 50), rng.integers(0, N, 50)
    np.testing.assert_allclose(orc.bwd_dw_at(X, dY, keep, BM, BK, p, r, c), dW[r, c], rtol=1e-13, atol=1e-13)


def test_bad_shapes_are_rejected():
    X, W, dY, keep, BM, BK, p = _case(seed=14)
    with pytest.raises(ValueError):
        orc.fwd(X, W, keep, BM + 1, BK, p)
    with pytest.raises(ValueError):
        orc.fwd(X, W, keep, BM, BK, 1.5)


def test_retiled_mask_gives_the_products_of_the_logical_mask():
    # Section 3.3: block splitting changes the tiling, not the result.  Logical blocks of 4 x 6
    # elements; forward with K-blocks halved, dW with M-blocks halved (the section's two uses), and both.
    MBL, KBL, LBM, LBK, N, p, seed = 3, 2, 4, 6, 5, 0.5, 6
    M, K = MBL * LBM, KBL * LBK
    X, W, dY = _rand((M, K), 1), _rand((K, N), 2), _rand((M, N), 3)
    logical = orc.mask(MBL, KBL, p, seed, 0)
    assert 0 < logical.sum() < logical.size
    ref = (orc.fwd(X, W, logical, LBM, LBK, p), orc.bwd_dx(dY, W, logical, LBM, LBK, p),
           orc.bwd_dw(X, dY, logical, LBM, LBK, p))
    for sm, sk in ((1, 2), (2, 1), (2, 3)):
        keep = orc.mask_split(MBL * sm, KBL * sk, sm, sk, p, seed, 0)
        BM, BK = LBM // sm, LBK // sk
        got = (orc.fwd(X, W, keep, BM, BK, p), orc.bwd_dx(dY, W, keep, BM, BK, p), orc.bwd_dw(X, dY, keep, BM, BK, p))
        for g, r in zip(got, ref):
            # the same elements are kept; only the grouping of the sums may differ
            assert np.allclose(g, r, rtol=1e-13, atol=1e-13), (sm, sk)


def test_weight_in_out_in_layout_by_index_loops_and_einsum():
    # Wt[N,K] is the transpose of Section 3.1's W[K,N].  Pins: scalar index loops on a tiny case (a missing or
    # doubled transpose, or a gradient left in [K,N], fails them), einsum with an element mask on non-square
    # and on square shapes (square shapes pass every shape check with the wrong orientation).
    rng = np.random.default_rng(5)
    for (M, K, N, BM, BK) in ((4, 6, 3, 2, 3), (6, 4, 4, 3, 2), (4, 4, 4, 2, 2)):
        X, Wt, dY = rng.standard_normal((M, K)), rng.standard_normal((N, K)), rng.standard_normal((M, N))
        keep = (rng.random((M // BM, K // BK)) < 0.6).astype(np.uint8)
        keep[0, 0] = 1
        p = 0.25
        s = 1.0 / (1.0 - p)
        el = np.repeat(np.repeat(keep, BM, axis=0), BK, axis=1).astype(np.float64)
        Y, dX, dWt = orc.fwd_wt(X, Wt, keep, BM, BK, p), orc.bwd_dx_wt(dY, Wt, keep, BM, BK, p), orc.bwd_dw_wt(X, dY, keep, BM, BK, p)
        assert Y.shape == (M, N) and dX.shape == (M, K) and dWt.shape == (N, K)
        for r in range(M):
            for n in range(N):
                assert abs(Y[r, n] - s * sum(X[r, k] * el[r, k] * Wt[n, k] for k in range(K))) < 1e-12
            for k in range(K):
                assert abs(dX[r, k] - s * el[r, k] * sum(dY[r, n] * Wt[n, k] for n in range(N))) < 1e-12
        for n in range(N):
            for k in range(K):
                assert abs(dWt[n, k] - s * sum(dY[r, n] * X[r, k] * el[r, k] for r in range(M))) < 1e-12
        assert np.allclose(Y, s * np.einsum("mk,nk->mn", X * el, Wt), atol=1e-12)
        assert np.allclose(dX, s * el * np.einsum("mn,nk->mk", dY, Wt), atol=1e-12)
        assert np.allclose(dWt, s * np.einsum("mn,mk->nk", dY, X * el), atol=1e-12)
        # and against the [K,N] functions on the transposed weight
        assert np.array_equal(Y, orc.fwd(X, np.ascontiguousarray(Wt.T), keep, BM, BK, p))
        assert np.array_equal(dWt.T, orc.bwd_dw(X, dY, keep, BM, BK, p))
