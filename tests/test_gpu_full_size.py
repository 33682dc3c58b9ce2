"""GPU parity at the full workload sizes, in the launch configuration the benchmark times.

Every element of Y, dX and dW is compared with the float64 oracle of arxiv 2411.01238
eq. (1)-(3) (whole products: a few seconds each on the host's cores, about half a minute for
the largest workload).  Two gates on the fp32-accumulated outputs: the parity tolerance
(relative Frobenius 1e-3, max-abs 5e-3 of max|ref|) and a regression gate two orders above
the error the kernels have (1e-5 for both measures: a 16-bit accumulation, a dropped slice
of a reduction or one wrong tile is far outside it).  16-bit outputs: fp16 to the parity
tolerance, bf16 as the rounding of an accurate result (half an ulp per entry).  The block
support of dX is compared with the oracle's keep flags.
"""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import WORKLOADS, make_inputs
from _util import f64, assert_close, assert_bf16_rounding_of, assert_tight

pytestmark = pytest.mark.gpu


def _expand(keep, BM, BK):
    return np.repeat(np.repeat(keep.astype(bool), BM, axis=0), BK, axis=1)


def _check_product(tag, name, fn, ref, is_bf16):
    """fn(out_dtype=...) against the whole reference; returns the 16-bit output (device)."""
    o32 = fn(out_dtype=torch.float32)
    o16 = fn(out_dtype=None)
    torch.cuda.synchronize()
    got = f64(o32)
    fro, mabs = assert_close(got, ref, "%s %s fp32 out" % (tag, name))
    assert_tight(got, ref, "%s %s fp32 out" % (tag, name))
    print("  %s %s: rel-Frobenius %.2e max-abs/max|ref| %.2e over %d elements" % (tag, name, fro, mabs, ref.size), flush=True)
    del got
    if is_bf16:
        assert torch.equal(o16, o32.to(torch.bfloat16)), "%s %s bf16 != RNE(fp32 out)" % (tag, name)
        assert_bf16_rounding_of(f64(o16), ref, "%s %s bf16 out" % (tag, name))
    else:
        assert_close(f64(o16), ref, "%s %s fp16 out" % (tag, name))
    return o32, o16


def _whole_parity(w, p, layer=0):
    tag = "%s p=%.1f layer %d" % (w.name, p, layer)
    print("full-size case", tag, flush=True)
    X, W, dY = make_inputs(w, layer=layer)
    m = sdrop.sdrop_mask(w.M, w.K, w.BM, w.BK, p, w.mask_seed, layer)
    keep = orc.mask(w.MB, w.KB, p, w.mask_seed, layer)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    is_bf16 = X.dtype == torch.bfloat16

    ref = orc.fwd(Xd, Wd, keep, w.BM, w.BK, p)
    Y32, Y16 = _check_product(tag, "Y", lambda **k: sdrop.sdrop_fwd(Xg, Wg, m, **k), ref, is_bf16)
    # the call the benchmark's step makes (mask and eq. 1 in one launch where the grid allows it): the same Y bit
    # for bit, and a mask object with the same header, bits and kept count
    Ys, ms = sdrop.sdrop_fwd_seeded(Xg, Wg, w.BM, w.BK, p, w.mask_seed, layer)
    torch.cuda.synchronize()
    assert torch.equal(Ys, Y16), tag + ": sdrop_fwd_seeded differs from sdrop_mask + sdrop_fwd"
    assert torch.equal(ms.buf[:256], m.buf[:256]) and torch.equal(ms.bits(), m.bits()), tag + ": mask objects differ"
    del Y32, Y16, Ys
    ref = orc.bwd_dx(dYd, Wd, keep, w.BM, w.BK, p)
    dX32, dX16 = _check_product(tag, "dX", lambda **k: sdrop.sdrop_bwd_dx(dYg, Wg, m, **k), ref, is_bf16)
    ref = orc.bwd_dw(Xd, dYd, keep, w.BM, w.BK, p)
    dW32, dW16 = _check_product(tag, "dW", lambda **k: sdrop.sdrop_bwd_dw(Xg, dYg, m, **k), ref, is_bf16)
    del ref, Xd, dYd
    # both gradients in one call (one launch where the shapes allow it) are the two calls, bit for bit
    bx, bw = sdrop.sdrop_bwd(dYg, Wg, Xg, m)
    torch.cuda.synchronize()
    assert torch.equal(bx, dX16) and torch.equal(bw, dW16), tag + ": sdrop_bwd differs from the separate calls"
    # the weight as [N,K] (read and written in place where the kernels have a form for it, else through a transposed
    # copy): the same bits
    Wt = Wg.t().contiguous()
    assert torch.equal(sdrop.sdrop_fwd_ex(Xg, Wt, m, w_layout=sdrop.W_NK), sdrop.sdrop_fwd(Xg, Wg, m)), tag + ": Y with W as [N,K]"
    assert torch.equal(sdrop.sdrop_bwd_dx_ex(dYg, Wt, m, w_layout=sdrop.W_NK), dX16), tag + ": dX with W as [N,K]"
    assert torch.equal(sdrop.sdrop_bwd_dw_ex(Xg, dYg, m, w_layout=sdrop.W_NK), dW16.t().contiguous()), tag + ": dW as [N,K]"
    del bx, bw, dW32, dW16, Wt

    # per block, dX is all +0 exactly where the oracle's mask drops the block
    keep_t = torch.from_numpy(keep.astype(bool)).cuda()
    for dX in (dX32, dX16):
        blocks = dX.view(w.MB, w.BM, w.KB, w.BK)
        nz = (blocks != 0).any(dim=3).any(dim=1)
        assert torch.equal(nz, keep_t), tag + ": dX block support differs from the mask"
        neg0 = torch.signbit(blocks).any(dim=3).any(dim=1) & ~keep_t
        assert not neg0.any().item()


CASES = [(w.name, p) for w in WORKLOADS.values() if w.name != "tiny" for p in w.ps]


@pytest.mark.parametrize("name,p", CASES)
def test_full_size_every_element(name, p):
    _whole_parity(WORKLOADS[name], p)


def test_mlp_other_layers_use_their_own_stream():
    _whole_parity(WORKLOADS["mlp"], 0.5, layer=3)


def test_mlp_four_layers_chained():
    # the 4-layer MLP as a chain: layer l+1 reads the 16-bit Y of layer l, the backward pass feeds dX of
    # layer l+1 to layer l as its dY (no activation in between).  Each product is checked against the
    # oracle on exactly the 16-bit operands the device used, so errors do not accumulate in the check.
    w = WORKLOADS["mlp"]
    p = 0.5
    print("full-size case mlp chain", flush=True)
    X0, _, dY_last = make_inputs(w, layer=0)
    Ws = [make_inputs(w, layer=l)[1].cuda() for l in range(w.layers)]
    masks = [sdrop.sdrop_mask(w.M, w.K, w.BM, w.BK, p, w.mask_seed, l) for l in range(w.layers)]
    keeps = [orc.mask(w.MB, w.KB, p, w.mask_seed, l) for l in range(w.layers)]
    acts = [X0.cuda()]
    for l in range(w.layers):
        acts.append(sdrop.sdrop_fwd(acts[l], Ws[l], masks[l]))
    grads = [None] * (w.layers + 1)
    grads[w.layers] = dY_last.cuda()
    dWs = [None] * w.layers
    for l in reversed(range(w.layers)):
        dWs[l] = sdrop.sdrop_bwd_dw(acts[l], grads[l + 1], masks[l])
        grads[l] = sdrop.sdrop_bwd_dx(grads[l + 1], Ws[l], masks[l])
    torch.cuda.synchronize()

    for l in range(w.layers):
        Xd, Wd, dYd = f64(acts[l]), f64(Ws[l]), f64(grads[l + 1])
        assert np.isfinite(Xd).all() and np.isfinite(dYd).all()
        assert_close(f64(acts[l + 1]), orc.fwd(Xd, Wd, keeps[l], w.BM, w.BK, p), "chain layer %d Y" % l)
        assert_close(f64(grads[l]), orc.bwd_dx(dYd, Wd, keeps[l], w.BM, w.BK, p), "chain layer %d dX" % l)
        assert_close(f64(dWs[l]), orc.bwd_dw(Xd, dYd, keeps[l], w.BM, w.BK, p), "chain layer %d dW" % l)


def test_sparse_block_operators_full_size():
    # the producing layer with bias + ReLU / GELU, and eq. (2) with the ReLU gate, at 4096^3: the oracle's
    # eq. (2) at scale 1 (the producing layer's product on the kept blocks) goes through its own tail
    w = WORKLOADS["square4096"]
    p = 0.5
    print("full-size case sparse block operators", flush=True)
    X, W, dY = make_inputs(w)
    m = sdrop.sdrop_mask(w.M, w.K, w.BM, w.BK, p, w.mask_seed, 0)
    keep = orc.mask(w.MB, w.KB, p, w.mask_seed, 0)
    g = torch.Generator(device="cpu")
    g.manual_seed(4242)
    b0 = torch.randn(w.K, generator=g, dtype=torch.float32) * 8.0
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Xd, Wd, dYd, b0d = f64(X), f64(W), f64(dY), f64(b0)
    kept = _expand(keep, w.BM, w.BK)
    keep_t = torch.from_numpy(keep.astype(bool)).cuda()

    z = orc.bwd_dx(dYd, Wd, keep, w.BM, w.BK, 0.0)          # H W0^T on kept blocks, s = 1
    for act in (sdrop.ACT_RELU, sdrop.ACT_GELU_TANH):
        ref = np.where(kept, sb.act(z + b0d[None, :], act), 0.0)
        o32 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=act, out_dtype=torch.float32)
        o16 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=act)
        torch.cuda.synchronize()
        assert_close(f64(o32), ref, "producer act %d fp32 out" % act)
        assert torch.equal(o16, o32.to(torch.bfloat16))
        assert_bf16_rounding_of(f64(o16), ref, "producer act %d bf16 out" % act)
        nz = (o16.view(w.MB, w.BM, w.KB, w.BK) != 0).any(dim=3).any(dim=1)
        assert torch.equal(nz, keep_t)
    del z
    ref = np.where(kept & (Xd > 0.0), orc.bwd_dx(dYd, Wd, keep, w.BM, w.BK, p), 0.0)
    o32 = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, relu_mask=Xg, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(f64(o32), ref, "gated dX fp32 out")
    assert_tight(f64(o32), ref, "gated dX fp32 out")
