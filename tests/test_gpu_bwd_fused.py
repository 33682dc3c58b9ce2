"""sdrop_bwd: eq. (2) and eq. (3) of arxiv 2411.01238 (Section 3.1) in one call, and in one launch
where the shapes allow it.  Against the float64 oracle through the C ABI, and bit for bit against
the two separate entry points, with the single launch switched on and off."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom
from _util import f64, assert_close, assert_bf16_rounding_of

pytestmark = pytest.mark.gpu

CASES = [
    # M, K, N, BM, BK, dtype, p, seed, dX kernel forced persistent
    (1024, 512, 512, 128, 128, "bf16", 0.5, 1, False),    # one launch: one kept block per dX tile, 8 dW tiles
    (1536, 256, 512, 128, 128, "f16", 0.3, 2, False),     # one launch; the dW part writes split fp32 planes, a summing pass follows
    (2560, 2560, 256, 128, 128, "bf16", 0.1, 3, True),    # one launch: dX tiles of two kept blocks, persistent form
    (2560, 2560, 256, 128, 128, "f16", 0.1, 13, False),   # one launch: dX tiles of two kept blocks, a workgroup per tile
    (1536, 1536, 512, 128, 128, "bf16", 0.0, 14, False),  # the same with nothing dropped and a split dW
    (4096, 1024, 256, 128, 128, "f16", 0.7, 4, False),    # one launch: more dX workgroups than kept blocks
    (512, 768, 328, 128, 128, "bf16", 0.3, 5, False),     # ragged N: two launches
    (384, 512, 256, 64, 64, "f16", 0.5, 6, False),        # 64 x 64 blocks, short kept lists: one launch, both a workgroup per tile
    (2048, 512, 256, 64, 64, "bf16", 0.3, 16, False),     # the same with dW split into parts and summed
    (4096, 256, 256, 64, 64, "bf16", 0.0, 17, False),     # 64 x 64 blocks, long kept lists (persistent dW): two launches
    (384, 512, 328, 64, 64, "f16", 0.5, 18, False),       # 64 x 64 blocks, ragged N: two launches
    (512, 512, 256, 128, 64, "bf16", 0.4, 7, False),      # 128 x 64 blocks: two launches
    (128, 128, 256, 128, 128, "bf16", 0.0, 8, False),     # a single block
]


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed,force", CASES)
def test_both_gradients_in_one_call(M, K, N, BM, BK, dtype, p, seed, force):
    print("bwd fused", M, K, N, BM, BK, dtype, p, seed, force, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    ref_dx = orc.bwd_dx(f64(dY), f64(W), keep, BM, BK, p)
    ref_dw = orc.bwd_dw(f64(X), f64(dY), keep, BM, BK, p)
    if force:
        sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, 0)
    try:
        for out_dtype in (torch.float32, None):
            sep_dx = sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=out_dtype)
            sep_dw = sdrop.sdrop_bwd_dw(Xg, dYg, m, out_dtype=out_dtype)
            for fused in (1, 0):
                sdrop.set_tuning(sdrop.TUNE_BWD_FUSED, fused)
                dx, dw = sdrop.sdrop_bwd(dYg, Wg, Xg, m, out_dtype=out_dtype)
                torch.cuda.synchronize()
                tag = "bwd(%d,%d,%d,%dx%d,%s) fused=%d out=%s" % (M, K, N, BM, BK, dtype, fused, out_dtype)
                assert torch.equal(dx, sep_dx), tag + ": dX differs from sdrop_bwd_dx"
                assert torch.equal(dw, sep_dw), tag + ": dW differs from sdrop_bwd_dw"
                if out_dtype == torch.float32 or X.dtype == torch.float16:
                    assert_close(f64(dx), ref_dx, tag + " dX")
                    assert_close(f64(dw), ref_dw, tag + " dW")
                else:
                    assert_bf16_rounding_of(f64(dx), ref_dx, tag + " dX")
                    assert_bf16_rounding_of(f64(dw), ref_dw, tag + " dW")
    finally:
        sdrop.set_tuning(sdrop.TUNE_BWD_FUSED, 1)
        sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT)


def test_everything_dropped_and_outputs_given():
    M, K, N = 512, 512, 256
    X, W, dY = make_custom(M, K, N, "bf16", seed=9)
    print("bwd fused p=1", flush=True)
    m = sdrop.sdrop_mask(M, K, 128, 128, 1.0, 0, 0)
    dx = torch.full((M, K), 7.0, dtype=torch.bfloat16, device="cuda")
    dw = torch.full((K, N), 7.0, dtype=torch.bfloat16, device="cuda")
    a, b = sdrop.sdrop_bwd(dY.cuda(), W.cuda(), X.cuda(), m, out_dx=dx, out_dw=dw)
    torch.cuda.synchronize()
    assert a is dx and b is dw
    for o in (dx, dw):
        assert torch.count_nonzero(o).item() == 0 and not torch.signbit(o).any().item()


@pytest.mark.parametrize("width", [128, 256])
def test_one_launch_for_64_blocks_with_either_dx_tile_width(width):
    M, K, N, B, p, seed = 1024, 768, 512, 64, 0.4, 21
    print("bwd fused 64-blocks width", width, flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=seed)
    m = sdrop.sdrop_mask(M, K, B, B, p, seed, 0)
    keep = orc.mask(M // B, K // B, p, seed, 0)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    sdrop.set_tuning(sdrop.TUNE_DX_TILE_WIDTH, width)
    try:
        dx, dw = sdrop.sdrop_bwd(dYg, Wg, Xg, m, out_dtype=torch.float32)
        assert torch.equal(dx, sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=torch.float32))
        assert torch.equal(dw, sdrop.sdrop_bwd_dw(Xg, dYg, m, out_dtype=torch.float32))
    finally:
        sdrop.set_tuning(sdrop.TUNE_DX_TILE_WIDTH, 0)
    assert_close(f64(dx), orc.bwd_dx(f64(dY), f64(W), keep, B, B, p), "dX 64-blocks width %d" % width)
    assert_close(f64(dw), orc.bwd_dw(f64(X), f64(dY), keep, B, B, p), "dW 64-blocks width %d" % width)
