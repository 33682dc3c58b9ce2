"""GPU parity at the full workload sizes, in the launch configuration the benchmark times.

The oracle cannot form whole products of these sizes in seconds, so it evaluates the same
definitions (arxiv 2411.01238 eq. (1)-(3)) at sampled output positions, spread over every
kind of position: kept and dropped blocks, first/last rows and columns of tiles.  Properties
that hold at any size are checked on the whole output: dropped blocks of dX are +0, kept
blocks are not, the bf16 output is the rounding of the fp32 output.
"""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import WORKLOADS, make_inputs
from _util import f64, assert_close, assert_bf16_rounding_of

pytestmark = pytest.mark.gpu


def _positions(rng, R, C, n, tr, tc):
    """n positions in an R x C matrix: random ones plus tile corners (tile tr x tc)."""
    r = rng.integers(0, R, n)
    c = rng.integers(0, C, n)
    edge_r = np.array([0, tr - 1, tr, R - 1, R - tr, R // 2])
    edge_c = np.array([0, tc - 1, tc, C - 1, C - tc, C // 2])
    er, ec = np.meshgrid(edge_r % R, edge_c % C)
    return np.concatenate([r, er.reshape(-1)]), np.concatenate([c, ec.reshape(-1)])


def _sampled_parity(w, p, layer=0, n=400, n_dw=96):
    tag = "%s p=%.1f layer %d" % (w.name, p, layer)
    print("full-size case", tag, flush=True)
    X, W, dY = make_inputs(w, layer=layer)
    m = sdrop.sdrop_mask(w.M, w.K, w.BM, w.BK, p, w.mask_seed, layer)
    keep = orc.mask(w.MB, w.KB, p, w.mask_seed, layer)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    rng = np.random.default_rng(1234)
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    is_bf16 = X.dtype == torch.bfloat16

    def gather(t, r, c):
        return t[torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()].cpu().to(torch.float64).numpy()

    def check(name, fn, oracle_at, a, b, R, C, tr, tc, count):
        r, c = _positions(rng, R, C, count, tr, tc)
        ref = oracle_at(a, b, keep, w.BM, w.BK, p, r, c)
        o32 = fn(out_dtype=torch.float32)
        o16 = fn(out_dtype=None)
        torch.cuda.synchronize()
        assert torch.isfinite(o32).all().item(), tag + " " + name
        # tolerances are relative to the whole result; sampled entries stand in for it
        assert_close(gather(o32, r, c), ref, "%s %s fp32 out (sampled)" % (tag, name))
        if is_bf16:
            assert torch.equal(o16, o32.to(torch.bfloat16)), "%s %s bf16 != RNE(fp32 out)" % (tag, name)
            assert_bf16_rounding_of(gather(o16, r, c), ref, "%s %s bf16 out (sampled)" % (tag, name))
        else:
            assert_close(gather(o16, r, c), ref, "%s %s fp16 out (sampled)" % (tag, name))
        return o32, o16

    check("Y", lambda **k: sdrop.sdrop_fwd(Xg, Wg, m, **k), orc.fwd_at, Xd, Wd, w.M, w.N, w.BM, 256, n)
    dX32, dX16 = check("dX", lambda **k: sdrop.sdrop_bwd_dx(dYg, Wg, m, **k), orc.bwd_dx_at, dYd, Wd,
                       w.M, w.K, w.BM, w.BK, n)
    dW32, dW16 = check("dW", lambda **k: sdrop.sdrop_bwd_dw(Xg, dYg, m, **k), orc.bwd_dw_at, Xd, dYd, w.K, w.N, w.BK, 256, n_dw)
    # both gradients in one call (one launch where the shapes allow it) are the two calls, bit for bit
    bx, bw = sdrop.sdrop_bwd(dYg, Wg, Xg, m)
    torch.cuda.synchronize()
    assert torch.equal(bx, dX16) and torch.equal(bw, dW16), tag + ": sdrop_bwd differs from the separate calls"
    del bx, bw, dW32, dW16

    # whole-output property: per block, dX is all +0 exactly where the block is dropped
    keep_t = torch.from_numpy(keep.astype(bool)).cuda()
    for dX in (dX32, dX16):
        blocks = dX.view(w.MB, w.BM, w.KB, w.BK)
        nz = (blocks != 0).any(dim=3).any(dim=1)
        assert torch.equal(nz, keep_t), tag + ": dX block support differs from the mask"
        neg0 = torch.signbit(blocks).any(dim=3).any(dim=1) & ~keep_t
        assert not neg0.any().item()


CASES = [(w.name, p) for w in WORKLOADS.values() if w.name != "tiny" for p in w.ps]


@pytest.mark.parametrize("name,p", CASES)
def test_full_size_sampled(name, p):
    _sampled_parity(WORKLOADS[name], p)


def test_mlp_other_layers_use_their_own_stream():
    w = WORKLOADS["mlp"]
    _sampled_parity(w, 0.5, layer=3, n=200, n_dw=48)


def test_mlp_four_layers_chained():
    # the 4-layer MLP as a chain: layer l+1 reads the 16-bit Y of layer l, the backward pass feeds dX of
    # layer l+1 to layer l as its dY (no activation in between).  Each product is checked against the
    # oracle on exactly the 16-bit operands the device used, so errors do not accumulate in the check.
    w = WORKLOADS["mlp"]
    p = 0.5
    print("full-size case mlp chain", flush=True)
    rng = np.random.default_rng(99)
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

    def gather(t, r, c):
        return t[torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()].cpu().to(torch.float64).numpy()

    for l in range(w.layers):
        Xd, Wd, dYd = f64(acts[l].cpu()), f64(Ws[l].cpu()), f64(grads[l + 1].cpu())
        assert np.isfinite(Xd).all() and np.isfinite(dYd).all()
        r, c = _positions(rng, w.M, w.N, 150, w.BM, 256)
        assert_close(gather(acts[l + 1], r, c), orc.fwd_at(Xd, Wd, keeps[l], w.BM, w.BK, p, r, c), "chain layer %d Y" % l)
        r, c = _positions(rng, w.M, w.K, 150, w.BM, w.BK)
        assert_close(gather(grads[l], r, c), orc.bwd_dx_at(dYd, Wd, keeps[l], w.BM, w.BK, p, r, c), "chain layer %d dX" % l)
        r, c = _positions(rng, w.K, w.N, 48, w.BK, 256)
        assert_close(gather(dWs[l], r, c), orc.bwd_dw_at(Xd, dYd, keeps[l], w.BM, w.BK, p, r, c), "chain layer %d dW" % l)


def test_sparse_block_operators_full_size_sampled():
    # the producing layer with bias + ReLU, and eq. (2) with the ReLU gate, at 4096^3: the oracle's
    # sampled eq. (2) values (s = 1 for the producer) go through its own tail, position by position
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
    rng = np.random.default_rng(77)
    r, c = _positions(rng, w.M, w.K, 400, w.BM, w.BK)
    kept = keep[r // w.BM, c // w.BK].astype(bool)

    def gather(t):
        return t[torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()].cpu().to(torch.float64).numpy()

    for act in (sdrop.ACT_RELU, sdrop.ACT_GELU_TANH):
        z = orc.bwd_dx_at(dYd, Wd, keep, w.BM, w.BK, 0.0, r, c)          # H W0^T on kept blocks, s = 1
        ref = np.where(kept, sb.act(z + b0d[c], act), 0.0)
        o32 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=act, out_dtype=torch.float32)
        o16 = sdrop.sdrop_producer(dYg, Wg, b0.cuda(), m, act=act)
        torch.cuda.synchronize()
        assert_close(gather(o32), ref, "producer act %d fp32 out (sampled)" % act)
        assert torch.equal(o16, o32.to(torch.bfloat16))
        assert_bf16_rounding_of(gather(o16), ref, "producer act %d bf16 out (sampled)" % act)
        nz = (o16.view(w.MB, w.BM, w.KB, w.BK) != 0).any(dim=3).any(dim=1)
        assert torch.equal(nz, torch.from_numpy(keep.astype(bool)).cuda())
    ref = np.where(kept & (Xd[r, c] > 0.0), orc.bwd_dx_at(dYd, Wd, keep, w.BM, w.BK, p, r, c), 0.0)
    o32 = sdrop.sdrop_bwd_dx_ex(dYg, Wg, m, relu_mask=Xg, out_dtype=torch.float32)
    plain = sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(gather(o32), ref, "gated dX fp32 out (sampled)")
    # whole-output property: the gated result is the plain one where the gate is open, +0 elsewhere
    assert torch.equal(o32, torch.where(Xg > 0, plain, torch.zeros_like(plain)))
