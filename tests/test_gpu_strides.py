"""Row-strided operands and outputs (leading dimensions, through the _ex entry points): a column
range of a wider matrix is used in place, for the three products of arxiv 2411.01238 eq. (1)-(3)
and their tails, against the float64 oracle; nothing outside the range is written."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom
from _util import f64, assert_close

pytestmark = pytest.mark.gpu


def _inside(t, left, right, fill=None):
    """A copy of t (or an uninitialised matrix of its shape) as a column range of a wider GPU matrix."""
    rows, cols = t.shape
    wide = torch.full((rows, left + cols + right), 7.0, dtype=t.dtype, device="cuda")
    view = wide[:, left:left + cols]
    if fill is None:
        view.copy_(t)
    return wide, view


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (512, 768, 328, 128, 128, "bf16", 0.3, 1),     # per-tile kernels with ragged edges
    (1024, 512, 512, 128, 128, "f16", 0.5, 2),     # persistent kernels
    (2048, 256, 264, 64, 64, "bf16", 0.5, 3),      # dW as split parts + summing pass into a strided output
    (1024, 1024, 256, 128, 64, "f16", 0.3, 4),     # dX tiles of several blocks
])
def test_strided_operands_and_outputs(M, K, N, BM, BK, dtype, p, seed):
    print("strides", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    _, Xv = _inside(X, 8, 24)
    _, Wv = _inside(W, 16, 0)
    _, dYv = _inside(dY, 0, 40)
    assert not Xv.is_contiguous() and Xv.data_ptr() % 16 == 0
    for out_dtype in (torch.float32, X.dtype):
        for name, fn, a, b, ref, shape in (
                ("Y", sdrop.sdrop_fwd, Xv, Wv, orc.fwd(Xd, Wd, keep, BM, BK, p), (M, N)),
                ("dX", sdrop.sdrop_bwd_dx, dYv, Wv, orc.bwd_dx(dYd, Wd, keep, BM, BK, p), (M, K)),
                ("dW", sdrop.sdrop_bwd_dw, Xv, dYv, orc.bwd_dw(Xd, dYd, keep, BM, BK, p), (K, N))):
            wide, out = _inside(torch.empty(shape, dtype=out_dtype), 16, 8, fill=False)
            got = fn(a, b, m, out_dtype=out_dtype, out=out)
            torch.cuda.synchronize()
            assert got is out
            tag = "strided %s out=%s (%d,%d,%d,%dx%d)" % (name, out_dtype, M, K, N, BM, BK)
            if out_dtype == torch.float32 or X.dtype == torch.float16:
                assert_close(f64(out), ref, tag)
            # the same call on contiguous copies gives the same bits
            assert torch.equal(out, fn(a.contiguous(), b.contiguous(), m, out_dtype=out_dtype)), tag + ": differs from the contiguous call"
            # columns outside the range keep their contents
            assert torch.all(wide[:, :16] == 7.0).item() and torch.all(wide[:, 16 + shape[1]:] == 7.0).item(), tag + ": wrote outside"


def test_strided_tail_and_gate():
    M, K, N, BM, BK, p, seed = 1024, 512, 256, 128, 128, 0.5, 9
    print("strides tail", flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    bK = torch.randn(K, generator=g)
    _, dYv = _inside(dY, 8, 8)
    _, Wv = _inside(W, 0, 16)
    # the gate must have the output's leading dimension: both live in matrices of the same width
    _, gate = _inside(X, 16, 32)
    wide, out = _inside(torch.empty((M, K), dtype=torch.float32), 16, 32, fill=False)
    wide16, out16 = _inside(torch.empty((M, K), dtype=torch.bfloat16), 16, 32, fill=False)
    ref = sb.bwd_dx_tail(f64(dY), f64(W), keep, BM, BK, p, False, f64(bK), sdrop.ACT_RELU, f64(X))
    sdrop.sdrop_bwd_dx_ex(dYv, Wv, m, act=sdrop.ACT_RELU, bias=bK.cuda(), relu_mask=gate, out_dtype=torch.float32, out=out)
    sdrop.sdrop_bwd_dx_ex(dYv, Wv, m, act=sdrop.ACT_RELU, bias=bK.cuda(), relu_mask=gate, out=out16)
    torch.cuda.synchronize()
    assert_close(f64(out), ref, "strided gated dX")
    assert torch.equal(out16, out.to(torch.bfloat16))
    assert torch.all(wide[:, :16] == 7.0).item() and torch.all(wide[:, 16 + K:] == 7.0).item()
    with pytest.raises(ValueError):
        sdrop.sdrop_bwd_dx_ex(dYv, Wv, m, relu_mask=X.cuda(), out=out16)      # gate contiguous, output strided
