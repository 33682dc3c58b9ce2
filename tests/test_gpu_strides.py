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


def _guards_ok(wide, left, cols):
    return torch.all(wide[:, :left] == 7.0).item() and torch.all(wide[:, left + cols:] == 7.0).item()


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (512, 768, 328, 128, 128, "bf16", 0.3, 1),     # ragged N
    (1024, 512, 512, 128, 128, "f16", 0.5, 2),     # persistent kernels, one-launch backward
    (2048, 256, 264, 64, 64, "bf16", 0.5, 3),      # dW as split parts
    (4096, 512, 256, 64, 64, "f16", 0.5, 4),       # one launch for 64 x 64 blocks
])
def test_backward_in_one_call_with_leading_dimensions(M, K, N, BM, BK, dtype, p, seed):
    # sdrop_bwd on column ranges of wider matrices (sdrop_bwd_ex): the contiguous call's bits, the oracle's values,
    # nothing written outside the ranges
    print("strides bwd", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    _, Xv = _inside(X, 8, 24)
    _, Wv = _inside(W, 16, 0)
    _, dYv = _inside(dY, 0, 40)
    for out_dtype in (torch.float32, X.dtype):
        wdx, odx = _inside(torch.empty((M, K), dtype=out_dtype), 16, 8, fill=False)
        wdw, odw = _inside(torch.empty((K, N), dtype=out_dtype), 8, 32, fill=False)
        a, b = sdrop.sdrop_bwd(dYv, Wv, Xv, m, out_dtype=out_dtype, out_dx=odx, out_dw=odw)
        ca, cb = sdrop.sdrop_bwd(dY.cuda(), W.cuda(), X.cuda(), m, out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert a is odx and b is odw
        assert torch.equal(odx, ca) and torch.equal(odw, cb), "strided sdrop_bwd differs from the contiguous call"
        assert _guards_ok(wdx, 16, K) and _guards_ok(wdw, 8, N), "sdrop_bwd wrote outside the column ranges"
        if out_dtype == torch.float32:
            assert_close(f64(odx), orc.bwd_dx(f64(dY), f64(W), keep, BM, BK, p), "strided sdrop_bwd dX")
            assert_close(f64(odw), orc.bwd_dw(f64(X), f64(dY), keep, BM, BK, p), "strided sdrop_bwd dW")


def test_producer_with_leading_dimensions():
    M, N0, K, BM, BK, p, seed = 1024, 320, 512, 128, 128, 0.5, 11
    print("strides producer", flush=True)
    Xunused, W0t, H = make_custom(M, K, N0, "bf16", seed=seed)      # H [M,N0]; W0t [K,N0]: one row per output feature
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    g = torch.Generator(device="cpu")
    g.manual_seed(6)
    b0 = torch.randn(K, generator=g)
    _, Hv = _inside(H, 8, 16)
    _, Wv = _inside(W0t, 24, 8)
    for out_dtype in (torch.float32, torch.bfloat16):
        wide, out = _inside(torch.empty((M, K), dtype=out_dtype), 16, 40, fill=False)
        widez, z = _inside(torch.empty((M, K), dtype=out_dtype), 16, 40, fill=False)
        got, gz = sdrop.sdrop_producer(Hv, Wv, b0.cuda(), m, act=sdrop.ACT_RELU, out_dtype=out_dtype, out=out, preact=z)
        ref, refz = sdrop.sdrop_producer(H.cuda(), W0t.cuda(), b0.cuda(), m, act=sdrop.ACT_RELU, out_dtype=out_dtype, preact=True)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "strided producer differs from the contiguous call"
        kept = torch.from_numpy(np.repeat(np.repeat(keep.astype(bool), BM, axis=0), BK, axis=1)).cuda()
        assert torch.equal(torch.where(kept, z, torch.zeros_like(z)), torch.where(kept, refz, torch.zeros_like(refz)))
        assert _guards_ok(wide, 16, K) and _guards_ok(widez, 16, K)
        if out_dtype == torch.float32:
            assert_close(f64(out), sb.producer(f64(H), f64(W0t), f64(b0), keep, BM, BK, sdrop.ACT_RELU), "strided producer")


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (512, 768, 328, 128, 128, "bf16", 0.3, 1),     # ragged N, non-square weight
    (1024, 512, 512, 128, 128, "f16", 0.5, 2),     # square weight: a missing transposition would pass every shape check
    (2048, 256, 264, 64, 64, "bf16", 0.5, 3),      # dW as split parts + summing pass, then the transposition
    (1024, 1024, 256, 128, 64, "f16", 0.3, 4),
    (1024, 1024, 512, 64, 64, "bf16", 0.5, 5),    # whole tile columns: the kernels that read and write [N,K] in place
    (2048, 1024, 768, 128, 128, "bf16", 0.5, 6),
    (2048, 2048, 256, 128, 128, "f16", 0.9, 7),
])
def test_weight_in_out_in_layout(M, K, N, BM, BK, dtype, p, seed):
    # eq. (1)-(3) with the weight stored as Wt[N,K] (w_layout = W_NK), against the oracle's functions for that
    # layout, every element; contiguous and as a column range of a wider matrix
    print("weight [N,K]", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    Wt = W.t().contiguous()                              # [N, K]
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    Xg, Wtg, dYg, Wg = X.cuda(), Wt.cuda(), dY.cuda(), W.cuda()
    Xd, Wtd, dYd = f64(X), f64(Wt), f64(dY)
    refs = {"Y": orc.fwd_wt(Xd, Wtd, keep, BM, BK, p), "dX": orc.bwd_dx_wt(dYd, Wtd, keep, BM, BK, p),
            "dWt": orc.bwd_dw_wt(Xd, dYd, keep, BM, BK, p)}
    _, Wtv = _inside(Wt, 8, 16)
    for out_dtype in (torch.float32, X.dtype):
        Y = sdrop.sdrop_fwd_ex(Xg, Wtg, m, out_dtype=out_dtype, w_layout=sdrop.W_NK)
        dX = sdrop.sdrop_bwd_dx_ex(dYg, Wtg, m, out_dtype=out_dtype, w_layout=sdrop.W_NK)
        dWt = sdrop.sdrop_bwd_dw_ex(Xg, dYg, m, out_dtype=out_dtype, w_layout=sdrop.W_NK)
        torch.cuda.synchronize()
        assert tuple(dWt.shape) == (N, K)
        if out_dtype == torch.float32 or X.dtype == torch.float16:
            for name, got in (("Y", Y), ("dX", dX), ("dWt", dWt)):
                assert_close(f64(got), refs[name], "[N,K] weight %s out=%s" % (name, out_dtype))
        # the same products through the [K,N] entry points on the transposed weight: the same bits
        assert torch.equal(Y, sdrop.sdrop_fwd(Xg, Wg, m, out_dtype=out_dtype))
        assert torch.equal(dX, sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=out_dtype))
        assert torch.equal(dWt, sdrop.sdrop_bwd_dw(Xg, dYg, m, out_dtype=out_dtype).t().contiguous())
        # strided weight in, strided gradient out
        assert torch.equal(Y, sdrop.sdrop_fwd_ex(Xg, Wtv, m, out_dtype=out_dtype, w_layout=sdrop.W_NK))
        assert torch.equal(dX, sdrop.sdrop_bwd_dx_ex(dYg, Wtv, m, out_dtype=out_dtype, w_layout=sdrop.W_NK))
        wide, out = _inside(torch.empty((N, K), dtype=out_dtype), 16, 24, fill=False)
        sdrop.sdrop_bwd_dw_ex(Xg, dYg, m, out_dtype=out_dtype, out=out, w_layout=sdrop.W_NK)
        torch.cuda.synchronize()
        assert torch.equal(out, dWt) and _guards_ok(wide, 16, K)
        # the calls that fuse steps, with the same layout: the mask drawn in the forward's launch, both gradients in one call
        Ys, ms = sdrop.sdrop_fwd_seeded(Xg, Wtg, BM, BK, p, seed, 0, out_dtype=out_dtype, w_layout=sdrop.W_NK)
        bx, bwt = sdrop.sdrop_bwd(dYg, Wtg, Xg, ms, out_dtype=out_dtype, w_layout=sdrop.W_NK)
        torch.cuda.synchronize()
        assert torch.equal(Ys, Y) and torch.equal(ms.buf[:256], m.buf[:256]) and torch.equal(ms.bits(), m.bits())
        assert torch.equal(bx, dX) and torch.equal(bwt, dWt)
        Ys2, _ = sdrop.sdrop_fwd_seeded(Xg, Wtv, BM, BK, p, seed, 0, out_dtype=out_dtype, w_layout=sdrop.W_NK)
        wide, out = _inside(torch.empty((N, K), dtype=out_dtype), 16, 24, fill=False)
        bx2, _ = sdrop.sdrop_bwd(dYg, Wtv, Xg, m, out_dtype=out_dtype, out_dw=out, w_layout=sdrop.W_NK)
        torch.cuda.synchronize()
        assert torch.equal(Ys2, Y) and torch.equal(bx2, dX) and torch.equal(out, dWt) and _guards_ok(wide, 16, K)
        # and the seeded forward on a column range of a wider X with the [K,N] weight
        _, Xv = _inside(X, 8, 8)
        Ys3, _ = sdrop.sdrop_fwd_seeded(Xv, Wg, BM, BK, p, seed, 0, out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert torch.equal(Ys3, Y)
    # a workspace sized for the [K,N] call is too small for the [N,K] one
    L = sdrop.lib()
    import ctypes
    epi = sdrop._epilogue(sdrop.SCALE_DROPOUT, sdrop.ACT_NONE, None, None, N, (M, N), X.dtype, w_layout=sdrop.W_NK)
    code = sdrop._DTYPES[X.dtype]
    need = L.sdrop_workspace_bytes_ex(sdrop.OP_FWD, M, K, N, BM, BK, code, code, ctypes.byref(epi))
    assert need == K * N * 2
    Y = torch.full((M, N), 3.0, dtype=X.dtype, device="cuda")
    vp = ctypes.c_void_p
    rc = L.sdrop_fwd_ex(vp(Xg.data_ptr()), vp(Wtg.data_ptr()), vp(m.buf.data_ptr()), vp(Y.data_ptr()), M, K, N, BM, BK, p,
                        code, code, None, 0, sdrop._stream(), ctypes.byref(epi))
    assert rc == sdrop.EWORKSPACE
    torch.cuda.synchronize()
    assert torch.all(Y == 3.0).item()
