"""GPU parity of the sparse operators around the dropout (arxiv 2411.01238, Section 4.3 closing
remark: sparse operators for the layer before the dropout as well) against the float64 CPU
oracle, through the C ABI: the element-wise tail of eq. (1) and eq. (2) (scale choice, bias,
ReLU / tanh-GELU, ReLU-backward gate), eq. (3) with the scale chosen, and the output-sparse
producing layer.

Bar as for the plain products: relative Frobenius error <= 1e-3 and max-abs error <= 5e-3 max|ref|
for fp32 and fp16 outputs; a bf16 output is the round-to-nearest-even of the library's own fp32
output and within half a bf16 ulp (plus the accumulation allowance) of the oracle.  The gate
(relu_mask > 0) is decided on the same 16-bit input values by both sides, so it is exact.
"""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom
from _util import f64, assert_close, assert_bf16_rounding_of

pytestmark = pytest.mark.gpu


def _expand(keep, BM, BK):
    return np.repeat(np.repeat(keep.astype(bool), BM, axis=0), BK, axis=1)


def _bias(n, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(7000 + seed)
    return torch.randn(n, generator=g, dtype=torch.float32)


def _check(o32, o16, ref, dtype, tag):
    assert_close(f64(o32), ref, tag + " fp32 out")
    if dtype == torch.float16:
        assert_close(f64(o16), ref, tag + " fp16 out")
    else:
        assert torch.equal(o16, o32.to(torch.bfloat16)), tag + ": bf16 output is not RNE of the fp32 output"
        assert_bf16_rounding_of(f64(o16), ref, tag + " bf16 out")


CASES = [
    # M, K, N, BM, BK, dtype, p, seed
    (512, 768, 328, 128, 128, "bf16", 0.3, 1),     # per-tile kernels: two N tiles with a ragged tail of 72; dX with a ragged reduction
    (384, 512, 264, 64, 64, "f16", 0.5, 2),        # 64-row tiles, ragged tail of 8
    (1024, 512, 512, 128, 128, "bf16", 0.5, 3),    # persistent kernels of all three products, one kept block per dX tile
    (1024, 1024, 256, 128, 64, "f16", 0.3, 4),     # dX tiles of several 64-column blocks
    (512, 512, 256, 64, 128, "bf16", 0.4, 5),      # 64-row blocks without ragged edges
    (256, 256, 8, 128, 128, "f16", 0.5, 6),        # smallest legal N
]


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", CASES)
@pytest.mark.parametrize("act", [sdrop.ACT_NONE, sdrop.ACT_RELU, sdrop.ACT_GELU_TANH, sdrop.ACT_GELU_ERF])
def test_fwd_and_dx_tails(M, K, N, BM, BK, dtype, p, seed, act):
    print("tail", M, K, N, BM, BK, dtype, p, seed, act, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    bN, bK = _bias(N, seed), _bias(K, seed + 50)
    tag = "tail(%d,%d,%d,%dx%d,%s,act=%d)" % (M, K, N, BM, BK, dtype, act)
    # every combination of scale, bias and gate that the entry points accept, two at a time
    for scale_mode, with_bias, with_gate in ((sdrop.SCALE_DROPOUT, True, False), (sdrop.SCALE_ONE, False, True),
                                              (sdrop.SCALE_ONE, True, True)):
        one = scale_mode == sdrop.SCALE_ONE
        kw = dict(scale_mode=scale_mode, act=act)
        # eq. (1) with the tail; the gate has the output's shape [M, N]: dY serves as it
        ref = sb.fwd_tail(Xd, Wd, keep, BM, BK, p, one, f64(bN) if with_bias else None, act, dYd if with_gate else None)
        o32 = sdrop.sdrop_fwd_ex(Xg, Wg, m, bias=bN.cuda() if with_bias else None, relu_mask=dYg if with_gate else None,
                                 out_dtype=torch.float32, **kw)
        o16 = sdrop.sdrop_fwd_ex(Xg, Wg, m, bias=bN.cuda() if with_bias else None, relu_mask=dYg if with_gate else None, **kw)
        _check(o32, o16, ref, X.dtype, tag + " fwd mode %d bias %d gate %d" % (scale_mode, with_bias, with_gate))
        # eq. (2) with the tail; the gate has the shape [M, K]: X serves as it
        ref = sb.bwd_dx_tail(dYd, Wd, keep, BM, BK, p, one, f64(bK) if with_bias else None, act, Xd if with_gate else None)
        o32 = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, bias=bK.cuda() if with_bias else None, relu_mask=Xg if with_gate else None,
                                    out_dtype=torch.float32, **kw)
        o16 = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, bias=bK.cuda() if with_bias else None, relu_mask=Xg if with_gate else None, **kw)
        _check(o32, o16, ref, X.dtype, tag + " dx mode %d bias %d gate %d" % (scale_mode, with_bias, with_gate))
        dropped = ~_expand(keep, BM, BK)
        for o in (o32, o16):
            d = f64(o)
            assert np.all(d[dropped] == 0.0) and not np.any(np.signbit(d[dropped])), tag + " dx dropped blocks"
    torch.cuda.synchronize()


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", CASES)
def test_dw_with_scale_one_and_producer(M, K, N, BM, BK, dtype, p, seed):
    print("tail dw/producer", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    tag = "(%d,%d,%d,%dx%d,%s)" % (M, K, N, BM, BK, dtype)
    for scale_mode in (sdrop.SCALE_DROPOUT, sdrop.SCALE_ONE):
        ref = sb.bwd_dw_scaled(Xd, dYd, keep, BM, BK, p, scale_mode == sdrop.SCALE_ONE)
        o32 = sdrop.sdrop_bwd_dw_ex(Xg, dYg, m, scale_mode=scale_mode, out_dtype=torch.float32)
        o16 = sdrop.sdrop_bwd_dw_ex(Xg, dYg, m, scale_mode=scale_mode)
        _check(o32, o16, ref, X.dtype, "dw_ex" + tag + " mode %d" % scale_mode)
    # the producing layer: H[M,N0] = dY's role, W0[K,N0] = W's role, one bias value per column of X
    b0 = _bias(K, seed + 90)
    for act in (sdrop.ACT_NONE, sdrop.ACT_RELU, sdrop.ACT_GELU_TANH, sdrop.ACT_GELU_ERF):
        ref = sb.producer(dYd, Wd, f64(b0), keep, BM, BK, act)
        o32 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=act, out_dtype=torch.float32)
        o16 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=act)
        _check(o32, o16, ref, X.dtype, "producer" + tag + " act %d" % act)
        d = f64(o16)
        dropped = ~_expand(keep, BM, BK)
        assert np.all(d[dropped] == 0.0) and not np.any(np.signbit(d[dropped]))
    ref = sb.producer(dYd, Wd, None, keep, BM, BK, sdrop.ACT_NONE)
    assert_close(f64(sdrop.sdrop_producer(dYg, Wg, None, m, out_dtype=torch.float32)), ref, "producer" + tag + " bare")
    torch.cuda.synchronize()


def test_tails_in_the_persistent_dx_kernel_with_several_blocks_per_tile():
    # by default that kernel is chosen only for launches with many tiles per CU; here it is forced
    M, K, N, BM, BK, p, seed = 1024, 1024, 256, 128, 64, 0.3, 14
    print("tail dx persistent groups", flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    bK = _bias(K, seed)
    sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, 0)
    try:
        for act in (sdrop.ACT_RELU, sdrop.ACT_GELU_TANH):
            ref = sb.bwd_dx_tail(f64(dY), f64(W), keep, BM, BK, p, False, f64(bK), act, f64(X))
            o32 = sdrop.sdrop_bwd_dx_ex(dY.cuda(), W.cuda(), m, act=act, bias=bK.cuda(), relu_mask=X.cuda(), out_dtype=torch.float32)
            o16 = sdrop.sdrop_bwd_dx_ex(dY.cuda(), W.cuda(), m, act=act, bias=bK.cuda(), relu_mask=X.cuda())
            _check(o32, o16, ref, X.dtype, "forced persistent dx act %d" % act)
    finally:
        sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT)


def test_gate_never_reads_dropped_blocks_and_no_tail_is_the_plain_call():
    M, K, N, BM, BK, p, seed = 512, 512, 256, 128, 128, 0.5, 33
    print("tail gate NaN / identity", flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    dropped = torch.from_numpy(~_expand(keep, BM, BK))
    Xn = X.clone()
    Xn[dropped] = float("nan")
    a = sdrop.sdrop_bwd_dx_ex(dY.cuda(), W.cuda(), m, relu_mask=X.cuda())
    b = sdrop.sdrop_bwd_dx_ex(dY.cuda(), W.cuda(), m, relu_mask=Xn.cuda())
    assert torch.equal(a, b) and torch.isfinite(b).all().item()
    # epi = NULL and an all-default tail are the plain entry points, bit for bit
    for ex, plain, args in ((sdrop.sdrop_fwd_ex, sdrop.sdrop_fwd, (X.cuda(), W.cuda())),
                            (sdrop.sdrop_bwd_dx_ex, sdrop.sdrop_bwd_dx, (dY.cuda(), W.cuda())),
                            (sdrop.sdrop_bwd_dw_ex, sdrop.sdrop_bwd_dw, (X.cuda(), dY.cuda()))):
        assert torch.equal(ex(*args, m), plain(*args, m))


@pytest.mark.parametrize("BM,BK,N", [(128, 128, 256), (64, 64, 136)])     # persistent kernels; per-tile kernels with ragged edges
def test_tails_with_everything_dropped_and_nothing_dropped(BM, BK, N):
    M, K = 4 * BM, 6 * BK
    print("tail p=0 / p=1", BM, BK, N, flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=77)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    bN, bK = _bias(N, 1).cuda(), _bias(K, 2).cuda()
    # everything dropped: a bias is not added where there is no block; eq. (1) sees an empty X, so only the tail is left
    m = sdrop.sdrop_mask(M, K, BM, BK, 1.0, 0, 0)
    none = np.zeros((M // BM, K // BK), dtype=np.uint8)
    for o in (sdrop.sdrop_producer(dYg, Wg, bK, m, act=sdrop.ACT_GELU_TANH),
              sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, bias=bK, act=sdrop.ACT_RELU, relu_mask=Xg)):
        assert torch.count_nonzero(o).item() == 0 and not torch.signbit(o).any().item()
    y = sdrop.sdrop_fwd_ex(Xg, Wg, m, bias=bN, act=sdrop.ACT_RELU, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = sb.fwd_tail(f64(X), f64(W), none, BM, BK, 1.0, False, f64(bN.cpu()), sdrop.ACT_RELU)
    assert np.array_equal(f64(y), np.broadcast_to(np.maximum(f64(bN.cpu()), 0.0), (M, N))) and np.array_equal(f64(y), ref)
    # nothing dropped: the producer is a dense layer with bias and activation
    m = sdrop.sdrop_mask(M, K, BM, BK, 0.0, 0, 0)
    allk = np.ones((M // BM, K // BK), dtype=np.uint8)
    o = sdrop.sdrop_producer(dYg, Wg, bK, m, act=sdrop.ACT_RELU, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(f64(o), np.maximum(f64(dY) @ f64(W).T + f64(bK.cpu()), 0.0), "dense producer")
    assert_close(f64(o), sb.producer(f64(dY), f64(W), f64(bK.cpu()), allk, BM, BK, sdrop.ACT_RELU), "dense producer vs oracle")


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", CASES[:5])
def test_gelu_gates_and_preactivation_output(M, K, N, BM, BK, dtype, p, seed):
    print("tail gelu gates", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    tag = "(%d,%d,%d,%dx%d,%s)" % (M, K, N, BM, BK, dtype)
    # eq. (2) times the GELU's derivative at a saved pre-activation (X stands in for it: values ~ N(0,1))
    for mode in (sdrop.GATE_GELU_TANH, sdrop.GATE_GELU_ERF):
        ref = sb.bwd_dx_tail(dYd, Wd, keep, BM, BK, p, relu_mask=Xd, gate_mode=mode)
        o32 = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, relu_mask=Xg, gate_mode=mode, out_dtype=torch.float32)
        o16 = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, relu_mask=Xg, gate_mode=mode)
        _check(o32, o16, ref, X.dtype, "gelu-gated dX" + tag + " mode %d" % mode)
        ref = sb.fwd_tail(Xd, Wd, keep, BM, BK, p, relu_mask=dYd, gate_mode=mode)
        o32 = sdrop.sdrop_fwd_ex(Xg, Wg, m, relu_mask=dYg, gate_mode=mode, out_dtype=torch.float32)
        _check(o32, sdrop.sdrop_fwd_ex(Xg, Wg, m, relu_mask=dYg, gate_mode=mode), ref, X.dtype, "gelu-gated Y" + tag + " mode %d" % mode)
    # the producing layer with its second output: the value before the activation, on the kept blocks only
    b0 = _bias(K, seed + 90)
    kept = _expand(keep, BM, BK)
    for out_dtype in (torch.float32, None):
        z = torch.full((M, K), 5.0, dtype=out_dtype or X.dtype, device="cuda")
        x, z2 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=sdrop.ACT_GELU_ERF, out_dtype=out_dtype, preact=z)
        torch.cuda.synchronize()
        assert z2 is z
        assert torch.equal(x, sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=sdrop.ACT_GELU_ERF, out_dtype=out_dtype))
        zr = sb.producer_preact(dYd, Wd, f64(b0), keep, BM, BK)
        zd = f64(z)
        assert np.all(zd[~kept] == 5.0), "pre-activation output wrote a dropped block"
        if out_dtype == torch.float32 or X.dtype == torch.float16:
            got = np.where(kept, zd, 0.0)
            assert_close(got, zr, "producer pre-activation" + tag)
        else:
            assert_bf16_rounding_of(np.where(kept, zd, 0.0), zr, "producer pre-activation bf16" + tag)


def test_kept_fraction_hint_changes_the_plan_not_the_result():
    # a mask built from the caller's bits with a density far from 1 - p: with and without the planning hint the
    # products are the oracle's, and equal to each other bit for bit
    M, K, N, BM, BK, p = 4096, 2048, 512, 128, 128, 0.5
    print("kept_fraction hint", flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=41)
    rng = np.random.default_rng(41)
    keep = (rng.random((M // BM, K // BK)) < 0.06).astype(np.uint8)       # 6 % kept although p says 50 %
    keep[0, 0] = 1
    bits = torch.from_numpy(orc.pack_bits(keep).view(np.int64)).cuda()
    m = sdrop.sdrop_mask_from_bits(M, K, BM, BK, p, bits)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    frac = float(keep.mean())
    for od in (torch.float32, torch.bfloat16):
        plain = (sdrop.sdrop_fwd(Xg, Wg, m, out_dtype=od), sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=od),
                 sdrop.sdrop_bwd_dw(Xg, dYg, m, out_dtype=od))
        hinted = (sdrop.sdrop_fwd_ex(Xg, Wg, m, out_dtype=od, kept_fraction=frac),
                  sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, out_dtype=od, kept_fraction=frac),
                  sdrop.sdrop_bwd_dw_ex(Xg, dYg, m, out_dtype=od, kept_fraction=frac))
        torch.cuda.synchronize()
        for a, b in zip(plain, hinted):
            assert torch.equal(a, b)
        if od == torch.float32:
            assert_close(f64(hinted[0]), orc.fwd(f64(X), f64(W), keep, BM, BK, p), "hinted Y")
            assert_close(f64(hinted[1]), orc.bwd_dx(f64(dY), f64(W), keep, BM, BK, p), "hinted dX")
            assert_close(f64(hinted[2]), orc.bwd_dw(f64(X), f64(dY), keep, BM, BK, p), "hinted dW")
