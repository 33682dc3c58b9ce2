"""GPU parity of the three products (arxiv 2411.01238 Section 3.1 eq. (1)-(3)) against the
float64 CPU oracle, through the C ABI.

Bar: relative Frobenius error <= 1e-3 and max-abs error <= 5e-3 * max|ref| for the
fp32-accumulated result (out_dtype fp32) and for fp16 outputs.  A bf16-stored output
cannot meet 1e-3 against an unrounded reference (rounding to 8 mantissa bits alone
costs about 1.7e-3), so bf16 outputs are held to: bit-equal to the round-to-nearest-even
of the library's own fp32 output, and each entry within half a bf16 ulp (plus the fp32
accumulation allowance) of the oracle value.
"""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import WORKLOADS, make_inputs, make_custom
from _util import f64, assert_close, assert_bf16_rounding_of, assert_tight

pytestmark = pytest.mark.gpu


def _expand(keep, BM, BK):
    return np.repeat(np.repeat(keep.astype(bool), BM, axis=0), BK, axis=1)


def _run_all(X, W, dY, m, out_dtype):
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    Y = sdrop.sdrop_fwd(Xg, Wg, m, out_dtype=out_dtype)
    dX = sdrop.sdrop_bwd_dx(dYg, Wg, m, out_dtype=out_dtype)
    dW = sdrop.sdrop_bwd_dw(Xg, dYg, m, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return Y, dX, dW


def _check_16bit_outputs(outs16, outs32, refs, dtype, tag):
    for name, o16, o32, ref in zip(("Y", "dX", "dW"), outs16, outs32, refs):
        if dtype == torch.float16:
            assert_close(f64(o16), ref, "%s %s fp16 out" % (tag, name))
        else:
            assert torch.equal(o16, o32.to(torch.bfloat16)), "%s %s: bf16 output is not RNE of the fp32 output" % (tag, name)
            assert_bf16_rounding_of(f64(o16), ref, "%s %s bf16 out" % (tag, name))


def _full_parity(X, W, dY, BM, BK, p, seed, stream, tag, keep=None):
    M, K = X.shape
    if keep is None:
        m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, stream)
        keep = orc.mask(M // BM, K // BK, p, seed, stream)
    else:
        bits = torch.from_numpy(orc.pack_bits(keep).view(np.int64)).cuda()
        m = sdrop.sdrop_mask_from_bits(M, K, BM, BK, p, bits)
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    refs = (orc.fwd(Xd, Wd, keep, BM, BK, p), orc.bwd_dx(dYd, Wd, keep, BM, BK, p),
            orc.bwd_dw(Xd, dYd, keep, BM, BK, p))
    outs32 = _run_all(X, W, dY, m, torch.float32)
    for name, o, ref in zip(("Y", "dX", "dW"), outs32, refs):
        assert_close(f64(o), ref, "%s %s fp32 out" % (tag, name))
        assert_tight(f64(o), ref, "%s %s fp32 out" % (tag, name))
    outs16 = _run_all(X, W, dY, m, None)
    _check_16bit_outputs(outs16, outs32, refs, X.dtype, tag)
    # dropped blocks of dX are +0 exactly, in both output types
    dropped = ~_expand(keep, BM, BK)
    for o in (outs32[1], outs16[1]):
        d = f64(o)
        assert np.all(d[dropped] == 0.0) and not np.any(np.signbit(d[dropped])), tag + " dX dropped blocks"
    return keep


def test_tiny_workload():
    w = WORKLOADS["tiny"]
    X, W, dY = make_inputs(w)
    print("gemm tiny", flush=True)
    keep = _full_parity(X, W, dY, w.BM, w.BK, 0.5, w.mask_seed, 0, "tiny")
    assert int(keep.sum()) == 10


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (512, 768, 328, 128, 128, "bf16", 0.3, 1),    # two N tiles, ragged tail of 72
    (512, 768, 328, 128, 128, "f16", 0.5, 2),
    (384, 512, 264, 64, 64, "f16", 0.5, 3),       # ragged tail of 8
    (384, 512, 520, 64, 128, "bf16", 0.4, 4),     # three N tiles
    (640, 320, 72, 128, 64, "bf16", 0.2, 5),      # N smaller than any tile
    (256, 384, 512, 64, 64, "bf16", 0.7, 6),
    (256, 256, 8, 128, 128, "f16", 0.5, 7),       # smallest legal N
    (2048, 256, 264, 64, 64, "bf16", 0.5, 8),     # few dW tiles, long columns: dW runs as split parts + reduce
    (1536, 256, 512, 128, 128, "f16", 0.3, 9),    # the same with 128-blocks and no ragged edge
    (128, 64 * 200, 256, 64, 64, "f16", 0.2, 10), # 200 block columns: fwd walks a kept list longer than 128 entries
    (64 * 300, 128, 256, 64, 64, "bf16", 0.1, 11),  # 300 block rows: dW walks long column lists (and splits them)
    (128 * 150, 128, 264, 128, 128, "bf16", 0.0, 12),  # the same, all kept, 128-blocks, ragged N
    (256, 128 * 140, 256, 128, 128, "bf16", 0.05, 13),  # fwd: 140 block columns with two slices each
    # dX as a persistent kernel (128-row blocks, N a multiple of 64)
    (1024, 1024, 256, 128, 64, "bf16", 0.3, 14),  # groups of two 64-column blocks, cut where the block row changes
    (2048, 512, 128, 128, 128, "f16", 0.9, 15),   # mostly zero fill: more workgroups than kept blocks
    (128, 128, 64, 128, 128, "bf16", 0.0, 16),    # a single block, a single slice
    (4096, 4096, 64, 128, 128, "bf16", 0.1, 17),  # 256-wide tiles of two kept blocks, one slice per tile
    (4096, 2048, 64, 128, 64, "f16", 0.1, 18),    # 256-wide tiles of four kept 64-column blocks
    (512, 4096, 192, 128, 128, "f16", 0.5, 19),   # three slices per tile, 4 x 32 blocks
])
def test_mid_sizes_every_element(M, K, N, BM, BK, dtype, p, seed):
    print("gemm mid", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    _full_parity(X, W, dY, BM, BK, p, seed, 0, "mid(%d,%d,%d,%dx%d,%s)" % (M, K, N, BM, BK, dtype))


def test_p0_is_plain_gemm_and_p1_is_zero():
    X, W, dY = make_custom(256, 384, 136, "bf16", seed=11)
    print("gemm p0/p1", flush=True)
    keep = _full_parity(X, W, dY, 128, 128, 0.0, 0, 0, "p=0")
    assert keep.all()
    m = sdrop.sdrop_mask(256, 384, 128, 128, 1.0, 0, 0)
    for o in _run_all(X, W, dY, m, torch.float32) + _run_all(X, W, dY, m, None):
        assert torch.count_nonzero(o).item() == 0 and not torch.signbit(o).any().item()


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (1024, 1024, 256, 128, 64, "bf16", 0.3, 14),  # groups of two 64-column blocks, cut where the block row changes
    (4096, 4096, 64, 128, 128, "bf16", 0.1, 17),  # groups of two 128-column blocks
    (4096, 2048, 64, 128, 64, "f16", 0.1, 18),    # groups of four 64-column blocks
    (384, 2048, 128, 128, 64, "bf16", 0.6, 20),   # groups of two, rows with few kept blocks: many cuts, zero fill
])
def test_dx_persistent_kernel_with_several_blocks_per_tile(M, K, N, BM, BK, dtype, p, seed):
    # by default this kernel is chosen only for launches with many tiles per CU; here it is forced
    print("gemm dx persistent groups", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, 0)
    try:
        _full_parity(X, W, dY, BM, BK, p, seed, 0, "dx-persistent(%d,%d,%d,%dx%d,%s)" % (M, K, N, BM, BK, dtype))
    finally:
        sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT)


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (1024, 1024, 256, 128, 128, "bf16", 0.4, 41),   # width 256: two kept blocks per tile; width 128: one
    (512, 1024, 192, 128, 64, "f16", 0.6, 42),      # width 256: four 64-column blocks per tile; width 128: two
    (384, 512, 136, 64, 64, "bf16", 0.3, 43),       # 64-row blocks, ragged reduction: per-tile kernels only
    (1024, 1024, 264, 128, 128, "bf16", 0.4, 44),   # ragged reduction (one valid 16-byte chunk in the last slice): the
                                                    # persistent kernel's loaders clear the rest of that slice in LDS
    (512, 1024, 184, 128, 64, "f16", 0.5, 45),      # the same with seven valid chunks and 64-column blocks
])
def test_dx_every_tile_width_and_kernel_form(M, K, N, BM, BK, dtype, p, seed):
    # the host normally picks the width of dX's tiles and the kernel form from the expected number of
    # kept blocks; here every combination is forced and must give the same dX, bit for bit
    print("gemm dx widths", M, K, N, BM, BK, dtype, p, seed, flush=True)
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    ref = orc.bwd_dx(f64(dY), f64(W), keep, BM, BK, p)
    outs = []
    try:
        for width in (0, 128, 256):
            for knob in (sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT, 0):
                sdrop.set_tuning(sdrop.TUNE_DX_TILE_WIDTH, width)
                sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, knob)
                o = sdrop.sdrop_bwd_dx(dY.cuda(), W.cuda(), m, out_dtype=torch.float32)
                torch.cuda.synchronize()
                assert_close(f64(o), ref, "dX width %d knob %d" % (width, knob))
                outs.append(o)
    finally:
        sdrop.set_tuning(sdrop.TUNE_DX_TILE_WIDTH, 0)
        sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT)
    # a tile's reduction order does not depend on its width or on the kernel form
    for o in outs[1:]:
        assert torch.equal(o, outs[0])


def test_retilings_of_one_logical_mask_give_the_same_products():
    # Section 3.3: logical blocks of 128 x 128, used as such, with the K-blocks halved (the section's
    # forward pass), with the M-blocks halved (its dW), and quartered; each against the oracle on
    # its own tiling, whose three results agree with each other on the CPU already
    M, K, N, p, seed = 1024, 768, 256, 0.4, 31
    X, W, dY = make_custom(M, K, N, "bf16", seed=seed)
    print("gemm retiled masks", flush=True)
    Xd, Wd, dYd = f64(X), f64(W), f64(dY)
    logical = orc.mask(M // 128, K // 128, p, seed, 0)
    ref = (orc.fwd(Xd, Wd, logical, 128, 128, p), orc.bwd_dx(dYd, Wd, logical, 128, 128, p),
           orc.bwd_dw(Xd, dYd, logical, 128, 128, p))
    for BM, BK in ((128, 128), (128, 64), (64, 128), (64, 64)):
        sm, sk = 128 // BM, 128 // BK
        m = sdrop.sdrop_mask_split(M, K, BM, BK, sm, sk, p, seed, 0)
        keep = orc.mask_split(M // BM, K // BK, sm, sk, p, seed, 0)
        torch.cuda.synchronize()
        assert np.array_equal(m.bits().cpu().numpy().view(np.uint64), orc.pack_bits(keep))
        outs = _run_all(X, W, dY, m, torch.float32)
        for name, o, r in zip(("Y", "dX", "dW"), outs, ref):
            assert_close(f64(o), r, "retiled %dx%d %s" % (BM, BK, name))


def test_p1_and_p0_without_ragged_edges():
    # the persistent kernels: everything dropped (zero fill only, no tile at all) and everything kept
    X, W, dY = make_custom(512, 512, 128, "bf16", seed=21)
    print("gemm p0/p1 persistent", flush=True)
    keep = _full_parity(X, W, dY, 128, 128, 0.0, 0, 0, "p=0 persistent")
    assert keep.all()
    m = sdrop.sdrop_mask(512, 512, 128, 128, 1.0, 0, 0)
    for o in _run_all(X, W, dY, m, torch.float32) + _run_all(X, W, dY, m, None):
        assert torch.count_nonzero(o).item() == 0 and not torch.signbit(o).any().item()


@pytest.mark.parametrize("B,N", [(64, 136), (128, 128)])    # per-tile kernels with a ragged edge; persistent kernels
def test_explicit_masks_all_dropped_rows_and_columns(B, N):
    X, W, dY = make_custom(6 * B, 6 * B, N, "f16", seed=12)
    print("gemm explicit masks", B, N, flush=True)
    BM = BK = B
    keep = np.ones((6, 6), dtype=np.uint8)
    keep[2, :] = 0          # an empty block row: those rows of Y are zero
    keep[:, 4] = 0          # an empty block column: those rows of dW are zero
    keep[0, 1] = 0
    _full_parity(X, W, dY, BM, BK, 0.25, 0, 0, "explicit", keep=keep)
    _full_parity(X, W, dY, BM, BK, 0.5, 0, 0, "all-dropped", keep=np.zeros((6, 6), dtype=np.uint8))
    one = np.zeros((6, 6), dtype=np.uint8)
    one[5, 0] = 1
    _full_parity(X, W, dY, BM, BK, 0.5, 0, 0, "one-block", keep=one)


def test_dropped_blocks_are_never_read():
    # NaN planted in the dropped blocks of X must not reach Y or dW (Section 3.2)
    X, W, dY = make_custom(512, 512, 264, "bf16", seed=13)
    print("gemm nan poison", flush=True)
    BM = BK = 128
    p = 0.5
    m = sdrop.sdrop_mask(512, 512, BM, BK, p, 3, 0)
    keep = orc.mask(4, 4, p, 3, 0)
    assert 0 < keep.sum() < 16
    Xp = X.clone()
    Xp[torch.from_numpy(~_expand(keep, BM, BK))] = float("nan")
    Y0, _, dW0 = _run_all(X, W, dY, m, torch.float32)
    Y1, _, dW1 = _run_all(Xp, W, dY, m, torch.float32)
    assert torch.equal(Y0, Y1) and torch.equal(dW0, dW1)


def test_results_are_bitwise_reproducible():
    X, W, dY = make_custom(512, 512, 264, "f16", seed=14)
    m = sdrop.sdrop_mask(512, 512, 64, 64, 0.3, 1, 0)
    a = _run_all(X, W, dY, m, torch.float32)
    b = _run_all(X, W, dY, m, torch.float32)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_mask_for_another_problem_writes_nothing():
    X, W, dY = make_custom(256, 256, 64, "f16", seed=15)
    m = sdrop.sdrop_mask(256, 256, 64, 64, 0.5, 0, 0)
    wrong = sdrop.sdrop_mask(256, 256, 128, 128, 0.5, 0, 0)
    wrong.BM = wrong.BK = 64            # lie to the binding; the device header still says 128
    wrong.buf = torch.cat([wrong.buf, torch.zeros(m.buf.numel(), dtype=torch.uint8, device="cuda")])
    out = torch.full((256, 64), 7.0, dtype=torch.float16, device="cuda")
    sdrop.sdrop_fwd(X.cuda(), W.cuda(), wrong, out=out)
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)


def test_status_word_reports_what_only_the_device_can_see():
    # a mask of another problem, and a drawn mask used with another dropout probability: the call returns OK (it only
    # enqueues), the kernels write nothing, and the status word says so; a mask built from bits goes with any p
    M, K, N, BM, BK = 1024, 512, 256, 128, 128
    X, W, dY = make_custom(M, K, N, "bf16", seed=17)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    sdrop.status(clear=True)
    m = sdrop.sdrop_mask(M, K, BM, BK, 0.5, 3, 1)
    good = sdrop.sdrop_fwd(Xg, Wg, m)
    assert sdrop.status(clear=True) == 0
    hdr = m.buf[:256].cpu().numpy()
    assert hdr[56:64].view(np.float64)[0] == 0.5 and hdr[64:72].view(np.uint64)[0] == 3 and hdr[72:80].view(np.uint64)[0] == 1
    # another p for the same object: every product refuses
    m.p = 0.25
    outs = {"Y": torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda"),
            "dX": torch.full((M, K), 7.0, dtype=torch.bfloat16, device="cuda"),
            "dW": torch.full((K, N), 7.0, dtype=torch.bfloat16, device="cuda")}
    sdrop.sdrop_fwd(Xg, Wg, m, out=outs["Y"])
    assert sdrop.status(clear=False) == sdrop.STATUS_MASK_MISMATCH
    assert sdrop.status(clear=True) == sdrop.STATUS_MASK_MISMATCH
    assert sdrop.status(clear=True) == 0
    sdrop.sdrop_bwd(dYg, Wg, Xg, m, out_dx=outs["dX"], out_dw=outs["dW"])
    assert sdrop.status(clear=True) == sdrop.STATUS_MASK_MISMATCH
    for n, o in outs.items():
        assert torch.all(o == 7.0).item(), n + " was written with a mask drawn for another p"
    m.p = 0.5
    assert torch.equal(sdrop.sdrop_fwd(Xg, Wg, m), good) and sdrop.status() == 0
    # a mask from the caller's bits carries no p: any p is taken, the scale follows the call
    keep = orc.mask(M // BM, K // BK, 0.5, 3, 1)
    bits = torch.from_numpy(orc.pack_bits(keep).view(np.int64)).cuda()
    mb = sdrop.sdrop_mask_from_bits(M, K, BM, BK, 0.25, bits)
    y = sdrop.sdrop_fwd(Xg, Wg, mb, out_dtype=torch.float32)
    assert sdrop.status() == 0
    assert_close(f64(y), orc.fwd(f64(X), f64(W), keep, BM, BK, 0.25), "mask from bits with its own p")
    # a foreign mask
    wrong = sdrop.sdrop_mask(M, K, 64, 64, 0.5, 0, 0)
    wrong.BM = wrong.BK = 128
    sdrop.sdrop_fwd(Xg, Wg, wrong, out=outs["Y"])
    assert sdrop.status() == sdrop.STATUS_MASK_MISMATCH and torch.all(outs["Y"] == 7.0).item()


def test_binding_reports_errors():
    X, W, dY = make_custom(256, 256, 64, "f16", seed=16)
    m = sdrop.sdrop_mask(256, 256, 64, 64, 0.5, 0, 0)
    with pytest.raises(sdrop.SdropError) as e:
        sdrop.sdrop_fwd(X.cuda(), W.cuda()[:, :60].contiguous(), m)      # N = 60
    assert e.value.code == sdrop.ESHAPE
    with pytest.raises(sdrop.SdropError):
        sdrop.sdrop_fwd(X.cuda()[:128].contiguous(), W.cuda(), m)         # mask is for M = 256
    with pytest.raises(sdrop.SdropError) as e:
        sdrop.sdrop_fwd(X.cuda().float(), W.cuda().float(), m)
    assert e.value.code == sdrop.EDTYPE


def _patterns(MB, KB):
    full_row = np.zeros((MB, KB), dtype=np.uint8); full_row[MB // 2, :] = 1
    full_col = np.zeros((MB, KB), dtype=np.uint8); full_col[:, KB - 1] = 1
    checker = ((np.add.outer(np.arange(MB), np.arange(KB)) % 2) == 0).astype(np.uint8)
    lower = (np.subtract.outer(np.arange(MB), np.arange(KB)) >= 0).astype(np.uint8)
    last = np.zeros((MB, KB), dtype=np.uint8); last[MB - 1, KB - 1] = 1
    all_but_one = np.ones((MB, KB), dtype=np.uint8); all_but_one[0, 0] = 0
    return {"one full block row": full_row, "one full block column": full_col, "checkerboard": checker,
            "lower triangle": lower, "only the last block": last, "all but the first block": all_but_one}


@pytest.mark.parametrize("force_groups", [False, True])
def test_structured_masks_on_a_grid_larger_than_the_chip(force_groups):
    # 24 x 20 blocks of 128 x 128: more block positions than CUs, so the persistent kernels run several
    # tiles per workgroup, with kept lists that are as unbalanced as they get (an empty row next to a
    # full one, a single column, a triangle).  Once with the default choice of dX kernel, once with
    # tiles of several blocks forced onto the persistent kernel.
    MB, KB, B, N = 24, 20, 128, 256
    X, W, dY = make_custom(MB * B, KB * B, N, "bf16", seed=41)
    sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, 0 if force_groups else 16)
    try:
        for name, keep in _patterns(MB, KB).items():
            print("gemm structured mask:", name, force_groups, flush=True)
            p = 1.0 - float(keep.mean())              # the scale that goes with this kept fraction; any p would do
            _full_parity(X, W, dY, B, B, p, 0, 0, name, keep=keep)
    finally:
        sdrop.set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT)


@pytest.mark.parametrize("M,K,N", [(512, 768, 256), (512, 768, 136), (2048, 256, 512)])
def test_mask_built_for_another_problem_writes_nothing(M, K, N):
    # every kernel compares the mask object's header with the call's shape before it trusts a list entry:
    # persistent kernels and the one-launch backward; per-tile kernels; dW as split parts with its summing pass
    import ctypes
    B = 128
    print("gemm foreign mask", M, K, N, flush=True)
    X, W, dY = make_custom(M, K, N, "bf16", seed=5)
    Xg, Wg, dYg = X.cuda(), W.cuda(), dY.cuda()
    other = sdrop.sdrop_mask(K, M, B, B, 0.5, 1, 0)           # the transposed problem: same size, different header
    buf = torch.zeros(2 * other.buf.numel(), dtype=torch.uint8, device="cuda")
    buf[:other.buf.numel()] = other.buf
    ws = torch.zeros(max(16, sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, B, B, X.dtype, X.dtype)), dtype=torch.uint8, device="cuda")
    L = sdrop.lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    outs = {n: torch.full(s, 3.0, dtype=torch.bfloat16, device="cuda") for n, s in (("Y", (M, N)), ("dX", (M, K)), ("dW", (K, N)))}
    common = (M, K, N, B, B, 0.5, sdrop.BF16, sdrop.BF16, ws.data_ptr(), ws.numel(), st)
    assert L.sdrop_fwd(Xg.data_ptr(), Wg.data_ptr(), buf.data_ptr(), outs["Y"].data_ptr(), *common) == sdrop.OK
    assert L.sdrop_bwd_dx(dYg.data_ptr(), Wg.data_ptr(), buf.data_ptr(), outs["dX"].data_ptr(), *common) == sdrop.OK
    assert L.sdrop_bwd_dw(Xg.data_ptr(), dYg.data_ptr(), buf.data_ptr(), outs["dW"].data_ptr(), *common) == sdrop.OK
    torch.cuda.synchronize()
    for n, o in outs.items():
        assert torch.all(o == 3.0).item(), n + " was written with a foreign mask"
    assert L.sdrop_bwd(dYg.data_ptr(), Wg.data_ptr(), Xg.data_ptr(), buf.data_ptr(), outs["dX"].data_ptr(), outs["dW"].data_ptr(), *common) == sdrop.OK
    torch.cuda.synchronize()
    for n in ("dX", "dW"):
        assert torch.all(outs[n] == 3.0).item(), n + " was written by sdrop_bwd with a foreign mask"
