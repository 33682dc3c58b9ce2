"""Pins for the oracle of the sparse operators around the dropout (CPU only).

The block  Z = H W0^T + b0,  X = m . act(Z),  Y = s X W  (arxiv 2411.01238, Section 4.3 closing
remark, on top of eq. (1)-(3) and the block mask of Section 3.2) is pinned against: automatic
differentiation of the same block written with library tensor operations, the library's own GELU,
identities of the activation, a hand-countable tiny case computed with scalar loops, and the
float64 C oracle of eq. (1)-(3) in the cases where the tail is the identity.  Shapes are never
square, so a transposed operand or a swapped index fails.
"""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _case(seed=0, MB=3, KB=5, BM=4, BK=2, N0=6, N=7, p=0.4):
    M, K = MB * BM, KB * BK
    H = _rand((M, N0), seed)
    W0 = _rand((K, N0), seed + 1)
    b0 = _rand((K,), seed + 2)
    W = _rand((K, N), seed + 3)
    dY = _rand((M, N), seed + 4)
    keep = orc.mask(MB, KB, p, seed, 0)
    assert 0 < keep.sum() < keep.size
    return H, W0, b0, W, dY, keep, BM, BK, p


def _torch_block(H, W0, b0, W, keep, BM, BK, p, kind):
    """The block with library operations; the mask goes in by repeat_interleave, not by kron."""
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    Ht, W0t, b0t, Wt = t(H), t(W0), t(b0), t(W)
    m = torch.tensor(keep, dtype=torch.float64).repeat_interleave(BM, 0).repeat_interleave(BK, 1)
    Z = torch.nn.functional.linear(Ht, W0t, b0t)
    A = torch.relu(Z) if kind == sb.ACT_RELU else torch.nn.functional.gelu(Z, approximate="tanh" if kind == sb.ACT_GELU_TANH else "none")
    Y = (A * m) @ Wt / (1.0 - p)
    return Ht, W0t, b0t, Wt, A * m, Y


@pytest.mark.parametrize("kind", [sb.ACT_RELU, sb.ACT_GELU_TANH, sb.ACT_GELU_ERF])
def test_forward_matches_library_ops(kind):
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=3)
    X, Y = sb.block_forward(H, W0, b0, W, keep, BM, BK, p, kind)
    _, _, _, _, Xt, Yt = _torch_block(H, W0, b0, W, keep, BM, BK, p, kind)
    np.testing.assert_allclose(X, Xt.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Y, Yt.detach().numpy(), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("kind", [sb.ACT_RELU, sb.ACT_GELU_TANH, sb.ACT_GELU_ERF])
def test_backward_matches_automatic_differentiation(kind):
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=5)
    g = sb.block_backward(H, W0, b0, W, keep, BM, BK, p, dY, kind)
    Ht, W0t, b0t, Wt, _, Yt = _torch_block(H, W0, b0, W, keep, BM, BK, p, kind)
    (Yt * torch.tensor(dY)).sum().backward()
    np.testing.assert_allclose(g["dH"], Ht.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dW0"], W0t.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["db0"], b0t.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g["dW"], Wt.grad.numpy(), rtol=1e-11, atol=1e-11)
    # the gradient at the pre-activation is zero on every dropped block
    m = np.repeat(np.repeat(keep, BM, 0), BK, 1)
    assert np.all(g["dZ"][m == 0] == 0.0)


def test_backward_pieces_are_the_three_products():
    """The backward of the producing layer is eq. (1) and eq. (3) with scale 1 applied to dZ,
    and dZ is eq. (2) gated by the ReLU output: the decomposition the fused entry points use."""
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=7)
    g = sb.block_backward(H, W0, b0, W, keep, BM, BK, p, dY)
    X, _ = sb.block_forward(H, W0, b0, W, keep, BM, BK, p, sb.ACT_RELU)
    dZ = sb.bwd_dx_tail(dY, W, keep, BM, BK, p, relu_mask=X)
    np.testing.assert_allclose(dZ, g["dZ"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.fwd_tail(dZ, W0, keep, BM, BK, p, scale_one=True), g["dH"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.bwd_dw_scaled(dZ, H, keep, BM, BK, p, scale_one=True), g["dW0"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.bwd_dw_scaled(X, dY, keep, BM, BK, p), g["dW"], rtol=1e-12, atol=1e-12)


def test_identity_tail_is_eq_1_to_3():
    """Without a tail the functions are the C oracle of eq. (1)-(3) (pinned on its own)."""
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=9)
    X = _rand((keep.shape[0] * BM, keep.shape[1] * BK), 21)
    np.testing.assert_allclose(sb.fwd_tail(X, W, keep, BM, BK, p), orc.fwd(X, W, keep, BM, BK, p), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.bwd_dx_tail(dY, W, keep, BM, BK, p), orc.bwd_dx(dY, W, keep, BM, BK, p), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.bwd_dw_scaled(X, dY, keep, BM, BK, p), orc.bwd_dw(X, dY, keep, BM, BK, p), rtol=1e-12, atol=1e-12)
    # the producer without bias and activation is eq. (2) at s = 1
    np.testing.assert_allclose(sb.producer(H, W0, None, keep, BM, BK), orc.bwd_dx(H, W0, keep, BM, BK, 0.0), rtol=1e-12, atol=1e-12)


def test_producer_by_scalar_loops():
    MB, KB, BM, BK, N0 = 2, 3, 2, 2, 3
    M, K = MB * BM, KB * BK
    H, W0, b0 = _rand((M, N0), 1), _rand((K, N0), 2), _rand((K,), 3)
    keep = np.array([[1, 0, 1], [0, 1, 1]], dtype=np.uint8)
    X = sb.producer(H, W0, b0, keep, BM, BK, sb.ACT_RELU)
    for r in range(M):
        for c in range(K):
            z = b0[c]
            for n in range(N0):
                z += H[r, n] * W0[c, n]
            want = max(z, 0.0) if keep[r // BM, c // BK] else 0.0
            assert abs(X[r, c] - want) < 1e-13


def test_gelu_tanh_identities():
    v = np.linspace(-6.0, 6.0, 241)
    g = sb.act(v, sb.ACT_GELU_TANH)
    ref = torch.nn.functional.gelu(torch.tensor(v), approximate="tanh").numpy()
    np.testing.assert_allclose(g, ref, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(g - sb.act(-v, sb.ACT_GELU_TANH), v, rtol=0, atol=1e-14)   # g(v) - g(-v) = v
    assert sb.act(np.array([0.0]), sb.ACT_GELU_TANH)[0] == 0.0
    assert abs(sb.act(np.array([10.0]), sb.ACT_GELU_TANH)[0] - 10.0) < 1e-12
    # close to the erf form it approximates
    from math import erf, sqrt
    exact = np.array([0.5 * x * (1.0 + erf(x / sqrt(2.0))) for x in v])
    assert np.max(np.abs(g - exact)) < 1e-3


def test_tail_order_and_gate():
    v = np.array([[-1.0, 0.5, 2.0, -0.25]])
    bias = np.array([0.5, -1.0, 0.0, 0.5])
    gate = np.array([[1.0, 1.0, 0.0, -0.0]])
    # bias first, then the activation, then the gate
    np.testing.assert_array_equal(sb.tail(v, bias, sb.ACT_RELU, gate), np.array([[0.0, 0.0, 0.0, 0.0]]))
    np.testing.assert_array_equal(sb.tail(v, bias, sb.ACT_NONE, gate), np.array([[-0.5, -0.5, 0.0, 0.0]]))
    np.testing.assert_array_equal(sb.tail(v, None, sb.ACT_RELU, None), np.array([[0.0, 0.5, 2.0, 0.0]]))


def test_dropped_blocks_of_inputs_are_not_read():
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=11)
    m = np.repeat(np.repeat(keep, BM, 0), BK, 1)
    X = _rand(m.shape, 31)
    Xn = X.copy()
    Xn[m == 0] = np.nan
    np.testing.assert_array_equal(sb.fwd_tail(Xn, W, keep, BM, BK, p, bias=_rand((W.shape[1],), 5), kind=sb.ACT_RELU),
                                  sb.fwd_tail(X, W, keep, BM, BK, p, bias=_rand((W.shape[1],), 5), kind=sb.ACT_RELU))
    out = sb.bwd_dx_tail(dY, W, keep, BM, BK, p, relu_mask=Xn)
    assert np.all(np.isfinite(out)) and np.all(out[m == 0] == 0.0)


def test_everything_dropped_or_kept():
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=13)
    none = np.zeros_like(keep)
    assert np.all(sb.producer(H, W0, b0, none, BM, BK, sb.ACT_GELU_TANH) == 0.0)
    allk = np.ones_like(keep)
    np.testing.assert_allclose(sb.producer(H, W0, b0, allk, BM, BK, sb.ACT_RELU), np.maximum(H @ W0.T + b0, 0.0), rtol=1e-13)
    assert sb.scale_of(1.0) == 0.0 and sb.scale_of(0.0) == 1.0 and sb.scale_of(0.75) == 4.0 and sb.scale_of(0.75, True) == 1.0


def test_gelu_erf_is_v_times_the_normal_cdf():
    from scipy.stats import norm
    v = np.linspace(-7.0, 7.0, 281)
    g = sb.act(v, sb.ACT_GELU_ERF)
    np.testing.assert_allclose(g, v * norm.cdf(v), rtol=1e-12, atol=1e-15)          # another library's route to Phi
    np.testing.assert_allclose(g, torch.nn.functional.gelu(torch.tensor(v)).numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(g - sb.act(-v, sb.ACT_GELU_ERF), v, rtol=0, atol=1e-14)
    assert sb.act(np.array([0.0]), sb.ACT_GELU_ERF)[0] == 0.0


@pytest.mark.parametrize("kind", [sb.ACT_RELU, sb.ACT_GELU_TANH, sb.ACT_GELU_ERF])
def test_activation_derivative_by_central_differences(kind):
    z = np.linspace(-5.0, 5.0, 401) + 0.0123            # keeps clear of the ReLU's kink at 0
    h = 1e-6
    fd = (sb.act(z + h, kind) - sb.act(z - h, kind)) / (2 * h)
    np.testing.assert_allclose(sb.act_grad(z, kind), fd, rtol=0, atol=2e-9)


@pytest.mark.parametrize("kind,mode", [(sb.ACT_GELU_TANH, sb.GATE_GELU_TANH), (sb.ACT_GELU_ERF, sb.GATE_GELU_ERF)])
def test_gelu_backward_pieces_are_the_three_products(kind, mode):
    """dZ of a GELU block is eq. (2) gated by the GELU's derivative at the saved pre-activation."""
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=17)
    g = sb.block_backward(H, W0, b0, W, keep, BM, BK, p, dY, kind)
    Zk = sb.producer_preact(H, W0, b0, keep, BM, BK)
    m = np.repeat(np.repeat(keep, BM, 0), BK, 1)
    np.testing.assert_allclose(Zk, np.where(m > 0, g["Z"], 0.0), rtol=1e-12, atol=1e-12)
    dZ = sb.bwd_dx_tail(dY, W, keep, BM, BK, p, relu_mask=Zk, gate_mode=mode)
    np.testing.assert_allclose(dZ, g["dZ"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.fwd_tail(dZ, W0, keep, BM, BK, p, scale_one=True), g["dH"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sb.bwd_dw_scaled(dZ, H, keep, BM, BK, p, scale_one=True), g["dW0"], rtol=1e-12, atol=1e-12)


def test_bias_gradient_counts_kept_rows_and_ignores_dropped_blocks():
    # dZ = 1 everywhere: column k sums to BM times the number of kept blocks in its block column
    MB, KB, BM, BK = 5, 3, 4, 2
    keep = orc.mask(MB, KB, 0.5, 3, 0)
    assert 0 < keep.sum() < keep.size
    got = sb.bias_grad(np.ones((MB * BM, KB * BK)), keep, BM, BK)
    np.testing.assert_array_equal(got, np.repeat(keep.sum(axis=0) * BM, BK))
    # scalar loops over a random dZ whose dropped blocks hold NaN
    dZ = _rand((MB * BM, KB * BK), 8)
    want = np.zeros(KB * BK)
    for r in range(MB * BM):
        for k in range(KB * BK):
            if keep[r // BM, k // BK]:
                want[k] += dZ[r, k]
            else:
                dZ[r, k] = np.nan
    np.testing.assert_allclose(sb.bias_grad(dZ, keep, BM, BK), want, rtol=1e-13, atol=1e-13)


def test_bias_gradient_is_the_blocks_derivative_by_central_differences():
    H, W0, b0, W, dY, keep, BM, BK, p = _case(seed=21)
    g = sb.block_backward(H, W0, b0, W, keep, BM, BK, p, dY, sb.ACT_GELU_ERF)
    np.testing.assert_allclose(g["db0"], sb.bias_grad(g["dZ"], keep, BM, BK), rtol=0, atol=0)
    eps = 1e-6
    for k in range(b0.size):
        e = np.zeros_like(b0); e[k] = eps
        lp = (sb.block_forward(H, W0, b0 + e, W, keep, BM, BK, p, sb.ACT_GELU_ERF)[1] * dY).sum()
        lm = (sb.block_forward(H, W0, b0 - e, W, keep, BM, BK, p, sb.ACT_GELU_ERF)[1] * dY).sum()
        assert abs((lp - lm) / (2 * eps) - g["db0"][k]) <= 1e-6 * max(1.0, abs(g["db0"][k])), k
