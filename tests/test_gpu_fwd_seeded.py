"""sdrop_fwd_seeded: the step's mask and eq. (1) (arxiv 2411.01238, Sections 3.1, 3.2, 3.4) in one launch.

Must be what sdrop_mask followed by sdrop_fwd gives, bit for bit: the mask object (header, bits, every index
list) and Y.  The mask object is also compared with lists derived from the oracle's keep flags, Y with the
oracle's product (every element at the mid sizes; the full-size workloads are covered bit-for-bit against the
two-call path, which tests/test_gpu_full_size.py compares with the oracle element by element).
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import WORKLOADS, make_inputs, make_custom
from _util import f64, assert_close, assert_tight, lists_from_keep

pytestmark = pytest.mark.gpu

LISTS = ("row_ptr", "col_idx", "blk_row", "col_ptr", "row_idx", "row_order", "col_order", "loc_row", "loc_col", "units")


def _same_object(a, b, tag):
    """Two mask objects hold the same header, bits and lists (the unused tails of the lists are not compared)."""
    assert torch.equal(a.buf[:256], b.buf[:256]), tag + ": headers differ"
    assert torch.equal(a.bits(), b.bits()), tag + ": bits differ"
    la, lb = a.lists(), b.lists()
    for k in LISTS:
        assert torch.equal(la[k], lb[k]), "%s: %s differs" % (tag, k)


def _against_keep(m, keep, tag):
    assert m.nnz() == int(keep.sum()), tag
    assert np.array_equal(m.bits().cpu().numpy().view(np.uint64), orc.pack_bits(keep)), tag + ": bits differ from the oracle's"
    got = {k: v.cpu().numpy() for k, v in m.lists().items()}
    want = lists_from_keep(keep)
    for k in want:
        assert np.array_equal(got[k], want[k]), "%s: %s differs from the oracle's flags" % (tag, k)
    MB, KB = keep.shape
    rc, cc = keep.sum(axis=1).astype(np.int64), keep.sum(axis=0).astype(np.int64)
    assert sorted(got["row_order"].tolist()) == list(range(MB)) and np.all(np.diff(rc[got["row_order"]]) <= 0)
    assert sorted(got["col_order"].tolist()) == list(range(KB)) and np.all(np.diff(cc[got["col_order"]]) <= 0)


def _case(X, W, BM, BK, p, seed, stream, tag, oracle_product=True, out_dtypes=(None, torch.float32)):
    print("fwd_seeded case", tag, flush=True)
    M, K = X.shape
    Xg, Wg = X.cuda(), W.cuda()
    keep = orc.mask(M // BM, K // BK, p, seed, stream)
    ref = orc.fwd(f64(X), f64(W), keep, BM, BK, p) if oracle_product else None
    for od in out_dtypes:
        # poison the mask buffer and the output: everything compared below was written by the call
        m1 = sdrop.Mask(M, K, BM, BK, p)
        m1.buf.fill_(0xA5)
        Y1 = torch.full((M, W.shape[1]), float("nan"), dtype=od or X.dtype, device="cuda")
        Y1, m1 = sdrop.sdrop_fwd_seeded(Xg, Wg, BM, BK, p, seed, stream, mask=m1, out_dtype=od, out=Y1)
        m2 = sdrop.sdrop_mask(M, K, BM, BK, p, seed, stream)
        Y2 = sdrop.sdrop_fwd(Xg, Wg, m2, out_dtype=od)
        torch.cuda.synchronize()
        _same_object(m1, m2, tag)
        _against_keep(m1, keep, tag)
        assert torch.equal(Y1, Y2), tag + ": Y differs from sdrop_mask + sdrop_fwd"
        if ref is not None and od == torch.float32:
            assert_close(f64(Y1), ref, tag + " Y fp32 out")
            assert_tight(f64(Y1), ref, tag + " Y fp32 out")
        # the object serves the backward calls of the step
        if od is None:
            dY = torch.ones_like(Y1)
            dx1, dw1 = sdrop.sdrop_bwd(dY, Wg, Xg, m1)
            dx2, dw2 = sdrop.sdrop_bwd(dY, Wg, Xg, m2)
            torch.cuda.synchronize()
            assert torch.equal(dx1, dx2) and torch.equal(dw1, dw2), tag + ": backward with the object differs"


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed,stream", [
    (256, 256, 256, 64, 64, "f16", 0.5, 0, 0),                 # the tiny workload: 4 x 4 blocks, fewer tiles than pieces
    (1024, 1024, 1000, 128, 128, "bf16", 0.5, 3, 1),           # ragged last tile column
    (640, 384, 264, 64, 64, "f16", 0.3, 4, 2),                 # 10 x 6 blocks, ragged
    (128, 8192, 512, 128, 128, "bf16", 0.5, 5, 3),             # one block row, 64 block columns (the widest grid)
    (8192, 2048, 256, 64, 64, "f16", 0.5, 6, 4),               # 128 x 32 blocks: the largest grid a workgroup draws
    (8192, 128, 512, 64, 128, "bf16", 0.2, 7, 5),              # 128 block rows, one block column
    (2048, 2048, 768, 128, 64, "bf16", 0.7, (1 << 63) + 12345, (1 << 40) + 7),     # 64-bit seed and stream
    (1536, 1152, 512, 128, 128, "f16", 0.0, 8, 0),             # nothing dropped
    (1536, 1152, 512, 128, 128, "f16", 1.0, 8, 0),             # everything dropped: Y = 0
    (2048, 3072, 256, 64, 64, "f16", 0.5, 9, 1),               # 32 x 48 blocks: 48 columns rounded up to 64 lanes
])
def test_seeded_forward_equals_mask_then_forward(M, K, N, BM, BK, dtype, p, seed, stream):
    X, W, _ = make_custom(M, K, N, dtype, seed=int(seed) % 1000)
    _case(X, W, BM, BK, p, seed, stream, "%dx%dx%d %dx%d %s p=%.1f" % (M, K, N, BM, BK, dtype, p))


@pytest.mark.parametrize("name,p,layer", [("square4096", 0.0, 0), ("square4096", 0.5, 0), ("square4096", 0.7, 0),
                                          ("mlp", 0.1, 0), ("mlp", 0.5, 3)])
def test_seeded_forward_on_the_workloads(name, p, layer):
    w = WORKLOADS[name]
    X, W, _ = make_inputs(w, layer=layer)
    _case(X, W, w.BM, w.BK, p, w.mask_seed, layer, "%s p=%.1f layer %d" % (name, p, layer), oracle_product=False,
          out_dtypes=(None,))


def test_largest_grid_and_grids_beyond_it():
    # 128 x 48 blocks (the FFN workload's grid, one launch); 128 x 64 (the largest a workgroup draws); a 256-row grid
    # and a 65-column grid (the two launches in turn): the same results
    for (M, K, N, BM, BK) in ((16384, 3072, 256, 128, 64), (8192, 4096, 256, 64, 64), (16384, 512, 256, 64, 128), (512, 8320, 256, 128, 128)):
        X, W, _ = make_custom(M, K, N, "bf16", seed=21)
        _case(X, W, BM, BK, 0.3, 11, 0, "fallback %dx%dx%d" % (M, K, N), oracle_product=False, out_dtypes=(None,))


def test_knob_off_gives_the_same_and_raw_c_abi_call():
    L = sdrop.lib()
    M, K, N, BM, BK, p = 1024, 1024, 512, 128, 128, 0.5
    X, W, _ = make_custom(M, K, N, "bf16", seed=31)
    Xg, Wg = X.cuda(), W.cuda()
    vp = ctypes.c_void_p
    outs = []
    for knob in (1, 0):
        sdrop.set_tuning(sdrop.TUNE_FWD_SEEDED, knob)
        try:
            m = sdrop.Mask(M, K, BM, BK, p)
            Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
            rc = L.sdrop_fwd_seeded(vp(Xg.data_ptr()), vp(Wg.data_ptr()), vp(m.buf.data_ptr()), m.buf.numel(), vp(Y.data_ptr()),
                                    M, K, N, BM, BK, p, 77, 5, sdrop.BF16, sdrop.BF16, sdrop._stream())
            assert rc == sdrop.OK
            torch.cuda.synchronize()
            outs.append((m, Y))
        finally:
            sdrop.set_tuning(sdrop.TUNE_FWD_SEEDED, 1)
    _same_object(outs[0][0], outs[1][0], "knob")
    assert torch.equal(outs[0][1], outs[1][1])
    _against_keep(outs[0][0], orc.mask(M // BM, K // BK, p, 77, 5), "raw call")
    # host-side errors: a mask buffer that is too small, a null output
    m = outs[0][0]
    Y = outs[0][1]
    assert L.sdrop_fwd_seeded(vp(Xg.data_ptr()), vp(Wg.data_ptr()), vp(m.buf.data_ptr()), 256, vp(Y.data_ptr()),
                              M, K, N, BM, BK, p, 77, 5, sdrop.BF16, sdrop.BF16, sdrop._stream()) == sdrop.EWORKSPACE
    assert L.sdrop_fwd_seeded(vp(Xg.data_ptr()), vp(Wg.data_ptr()), None, m.buf.numel(), vp(Y.data_ptr()),
                              M, K, N, BM, BK, p, 77, 5, sdrop.BF16, sdrop.BF16, sdrop._stream()) == sdrop.EINVAL
