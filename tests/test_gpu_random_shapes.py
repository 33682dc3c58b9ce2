"""Every-element parity of the three products (arxiv 2411.01238 Section 3.1 eq. (1)-(3)) on a seeded
sample of small shapes that lands on every kernel form: 64- and 128-row blocks, N with and without
ragged edges (per-tile and persistent kernels), few and many block columns (dW with and without
split reduction), sparsities from nothing to almost everything dropped."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom
from _util import f64, assert_close

pytestmark = pytest.mark.gpu


def _cases():
    rng = np.random.default_rng(20241101)
    out = []
    for n in range(36):
        BM, BK = (int(rng.choice([64, 128])) for _ in range(2))
        MB, KB = int(rng.integers(1, 13)), int(rng.integers(1, 13))
        # N: multiples of 256 / 64 (no ragged edge anywhere), of 8 (ragged), small and large
        N = int(rng.choice([64, 128, 192, 256, 512, 8, 72, 264, 328, 1024]))
        p = float(rng.choice([0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 0.97]))
        dtype = str(rng.choice(["bf16", "f16"]))
        out.append((MB * BM, KB * BK, N, BM, BK, dtype, p, 100 + n))
    return out


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", _cases())
def test_random_shape(M, K, N, BM, BK, dtype, p, seed):
    print("gemm random", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 1)
    keep = orc.mask(M // BM, K // BK, p, seed, 1)
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Y = sdrop.sdrop_fwd(Xg, Wg, m, out_dtype=torch.float32)
    dX = sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=torch.float32)
    dW = sdrop.sdrop_bwd_dw(Xg, dYg, m, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert m.nnz() == int(keep.sum())
    tag = "random(%d,%d,%d,%dx%d,%s,p=%.2f)" % (M, K, N, BM, BK, dtype, p)
    assert_close(f64(Y), orc.fwd(Xd, Wd, keep, BM, BK, p), tag + " Y")
    assert_close(f64(dX), orc.bwd_dx(dYd, Wd, keep, BM, BK, p), tag + " dX")
    assert_close(f64(dW), orc.bwd_dw(Xd, dYd, keep, BM, BK, p), tag + " dW")
    # 16-bit outputs of the same calls are the rounding of the fp32 ones
    Y16 = sdrop.sdrop_fwd(Xg, Wg, m)
    dX16 = sdrop.sdrop_bwd_dx(dYg, Wg, m)
    dW16 = sdrop.sdrop_bwd_dw(Xg, dYg, m)
    torch.cuda.synchronize()
    for a16, a32 in ((Y16, Y), (dX16, dX), (dW16, dW)):
        assert torch.equal(a16, a32.to(a16.dtype)), tag + ": 16-bit output is not the rounding of the fp32 output"
    # both gradients in one call are the two calls, bit for bit, whichever way they are launched
    bx, bw = sdrop.sdrop_bwd(dYg, Wg, Xg, m)
    assert torch.equal(bx, dX16) and torch.equal(bw, dW16), tag + ": sdrop_bwd differs from the separate calls"
    # one tail per case on eq. (1) and eq. (2), chosen by the seed: every kernel form meets every tail over the sample
    act = (sdrop.ACT_NONE, sdrop.ACT_RELU, sdrop.ACT_GELU_TANH)[seed % 3]
    one = bool(seed % 2)
    g = torch.Generator(device="cpu")
    g.manual_seed(9000 + seed)
    bN, bK = torch.randn(N, generator=g), torch.randn(K, generator=g)
    kw = dict(scale_mode=sdrop.SCALE_ONE if one else sdrop.SCALE_DROPOUT, act=act, out_dtype=torch.float32)
    Yt = sdrop.sdrop_fwd_ex(Xg, Wg, m, bias=bN.cuda(), relu_mask=dYg, **kw)
    dXt = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, bias=bK.cuda(), relu_mask=Xg, **kw)
    torch.cuda.synchronize()
    assert_close(f64(Yt), sb.fwd_tail(Xd, Wd, keep, BM, BK, p, one, f64(bN), act, dYd), tag + " Y with tail")
    assert_close(f64(dXt), sb.bwd_dx_tail(dYd, Wd, keep, BM, BK, p, one, f64(bK), act, Xd), tag + " dX with tail")
