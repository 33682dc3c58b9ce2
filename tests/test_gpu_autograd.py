"""The autograd wrapper must hand eq. (1)-(3) of arxiv 2411.01238 (Section 3.1) to torch unchanged:
forward and both gradients against the float64 oracle, with the mask the wrapper drew."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd.autograd import sparsedrop_matmul, SparseDropLinear, sparse_relu_block, sparse_act_block
from paper_2411_01238_amd.workloads import make_custom
from _util import f64, assert_close

pytestmark = pytest.mark.gpu


def test_function_matches_oracle_forward_and_gradients():
    M, K, N, BM, BK, p, seed, stream = 512, 384, 256, 128, 64, 0.4, 5, 2
    X, W, dY = make_custom(M, K, N, "f16", seed=3)
    x = X.cuda().requires_grad_(True)
    w = W.cuda().requires_grad_(True)
    y = sparsedrop_matmul(x, w, p, BM, BK, seed, stream)
    y.backward(dY.cuda())
    torch.cuda.synchronize()
    keep = orc.mask(M // BM, K // BK, p, seed, stream)
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    assert_close(f64(y.detach()), orc.fwd(Xd, Wd, keep, BM, BK, p), "autograd Y")
    assert_close(f64(x.grad), orc.bwd_dx(dYd, Wd, keep, BM, BK, p), "autograd dX")
    assert_close(f64(w.grad), orc.bwd_dw(Xd, dYd, keep, BM, BK, p), "autograd dW")


@pytest.mark.parametrize("N", [256, 136])        # the weight read in place / through a transposed copy
def test_function_with_the_weight_as_out_in(N):
    M, K, BM, BK, p, seed, stream = 512, 384, 128, 128, 0.4, 5, 2
    X, W, dY = make_custom(M, K, N, "bf16", seed=4)
    x = X.cuda().requires_grad_(True)
    wt = W.t().contiguous().cuda().requires_grad_(True)          # [N, K]
    y = sparsedrop_matmul(x, wt, p, BM, BK, seed, stream, weight_layout="nk")
    y.backward(dY.cuda())
    x2 = X.cuda().requires_grad_(True)
    w2 = W.cuda().requires_grad_(True)
    y2 = sparsedrop_matmul(x2, w2, p, BM, BK, seed, stream)
    y2.backward(dY.cuda())
    torch.cuda.synchronize()
    assert tuple(wt.grad.shape) == (N, K)
    assert torch.equal(y, y2) and torch.equal(x.grad, x2.grad) and torch.equal(wt.grad, w2.grad.t())
    keep = orc.mask(M // BM, K // BK, p, seed, stream)
    ref = orc.bwd_dw_wt(f64(X), f64(dY), keep, BM, BK, p)
    got = f64(wt.grad)
    assert np.max(np.abs(got - ref)) <= 2.0 ** -7 * np.max(np.abs(ref))          # a bf16 output: its rounding only


def test_module_with_a_linear_layers_state():
    lin = torch.nn.Linear(256, 384, bias=True).to(device="cuda", dtype=torch.bfloat16)
    layer = SparseDropLinear(256, 384, p=0.5, BM=128, BK=128, bias=True, seed=1, weight_layout="nk")
    layer.load_state_dict(lin.state_dict())              # same parameter names and shapes
    layer.eval()
    x = torch.randn(256, 256, device="cuda", dtype=torch.bfloat16)
    ref = f64(x) @ f64(lin.weight.detach()).T + f64(lin.bias.detach())
    assert_close(f64(layer(x).detach()), ref, "module in eval mode = the linear layer", rel_fro=5e-3, max_abs=2e-2)


def test_module_train_and_eval():
    torch.manual_seed(0)
    layer = SparseDropLinear(256, 128, p=0.5, BM=64, BK=64, bias=True, seed=9, dtype=torch.float16)
    x = torch.randn(4, 64, 256, device="cuda", dtype=torch.float16)      # leading dimensions are flattened
    layer.train()
    y0 = layer(x)
    y1 = layer(x)
    assert y0.shape == (4, 64, 128)
    assert not torch.equal(y0, y1)                     # a new mask per call
    keep = orc.mask(256 // 64, 256 // 64, 0.5, 9, 0)   # the first call used rng_stream 0
    ref = orc.fwd(f64(x.reshape(-1, 256)), f64(layer.weight.detach()), keep, 64, 64, 0.5)
    got = f64((y0 - layer.bias).detach().reshape(-1, 128))
    assert_close(got, ref, "module forward, first call")
    layer.eval()
    ye = layer(x)
    dense = f64(x.reshape(-1, 256)) @ f64(layer.weight.detach())
    assert_close(f64((ye - layer.bias).detach().reshape(-1, 128)), dense, "module eval = dense")
    y0.sum().backward()
    assert layer.weight.grad is not None and layer.bias.grad is not None


@pytest.mark.parametrize("act,kind", [("relu", sb.ACT_RELU), ("gelu", sb.ACT_GELU_ERF), ("gelu_tanh", sb.ACT_GELU_TANH)])
def test_sparse_block_matches_oracle_forward_and_gradients(act, kind):
    # Linear -> ReLU -> SparseDrop -> Linear with all six GEMMs sparse, against the chain rule
    # written out in float64.  The GPU keeps the hidden activation in 16 bits and gates the backward
    # on it; the oracle gates on its own float64 pre-activation: the two can differ only where that
    # pre-activation is within rounding of zero, so those few entries are left out of the max-abs
    # bound of dZ's consumers by comparing in the Frobenius norm only.
    M, N0, K, N, BM, BK, p, seed, stream = 512, 256, 384, 136, 128, 64, 0.4, 11, 3
    g = torch.Generator(device="cpu")
    g.manual_seed(123)
    H = (torch.randn(M, N0, generator=g)).to(torch.bfloat16)
    W0 = (torch.randn(K, N0, generator=g) / N0 ** 0.5).to(torch.bfloat16)
    b0 = torch.randn(K, generator=g) * 0.5
    W = (torch.randn(K, N, generator=g) / K ** 0.5).to(torch.bfloat16)
    dY = torch.randn(M, N, generator=g).to(torch.bfloat16)
    print("autograd sparse block", act, flush=True)
    h = H.cuda().requires_grad_(True)
    w0 = W0.cuda().requires_grad_(True)
    b = b0.cuda().requires_grad_(True)
    w = W.cuda().requires_grad_(True)
    y = sparse_act_block(h, w0, b, w, p, act, BM, BK, seed, stream)
    if act == "relu":
        assert torch.equal(y, sparse_relu_block(h, w0, b, w, p, BM, BK, seed, stream))
    y.backward(dY.cuda())
    torch.cuda.synchronize()
    keep = orc.mask(M // BM, K // BK, p, seed, stream)
    Hd, W0d, b0d, Wd, dYd = f64(H), f64(W0), f64(b0), f64(W), f64(dY)
    _, Yref = sb.block_forward(Hd, W0d, b0d, Wd, keep, BM, BK, p, kind)
    gref = sb.block_backward(Hd, W0d, b0d, Wd, keep, BM, BK, p, dYd, kind)
    # two 16-bit roundings on the way (X, then Y or a gradient): 2^-9 relative each in bf16
    tol = dict(rel_fro=6e-3, max_abs=3e-2)
    assert_close(f64(y.detach()), Yref, "block Y", **tol)
    assert_close(f64(w.grad), gref["dW"], "block dW", **tol)
    for name, got in (("dH", h.grad), ("dW0", w0.grad), ("db0", b.grad)):
        got = f64(got)
        assert np.all(np.isfinite(got))
        fro = np.linalg.norm(got - gref[name]) / np.linalg.norm(gref[name])
        assert fro <= 6e-3, "block %s: relative Frobenius error %.3e" % (name, fro)
    assert b.grad.dtype == torch.float32
