"""The autograd wrapper must hand eq. (1)-(3) of arxiv 2411.01238 (Section 3.1) to torch unchanged:
forward and both gradients against the float64 oracle, with the mask the wrapper drew."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd.autograd import sparsedrop_matmul, SparseDropLinear
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
