"""GPU parity: the device mask (Section 3.2 of arxiv 2411.01238, this build's Philox rule)
must equal the CPU oracle's bit for bit, and every index list must describe that same set."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import WORKLOADS
from _util import lists_from_keep

pytestmark = pytest.mark.gpu


def _check_mask(m, keep):
    MB, KB = keep.shape
    torch.cuda.synchronize()
    assert m.nnz() == int(keep.sum())
    got_bits = m.bits().cpu().numpy().view(np.uint64)
    assert np.array_equal(got_bits, orc.pack_bits(keep))
    got = {k: v.cpu().numpy() for k, v in m.lists().items()}
    want = lists_from_keep(keep)
    for k in ("row_ptr", "col_idx", "blk_row", "col_ptr", "row_idx", "loc_row", "loc_col"):
        assert np.array_equal(got[k], want[k]), k
    # the schedules are permutations sorted by descending kept count (ties: any order)
    rc, cc = keep.sum(axis=1).astype(np.int64), keep.sum(axis=0).astype(np.int64)
    assert sorted(got["row_order"].tolist()) == list(range(MB))
    assert sorted(got["col_order"].tolist()) == list(range(KB))
    assert np.all(np.diff(rc[got["row_order"]]) <= 0)
    assert np.all(np.diff(cc[got["col_order"]]) <= 0)


CASES = []
for w in WORKLOADS.values():
    for p in w.ps:
        for layer in range(w.layers):
            CASES.append((w.name, p, layer))


@pytest.mark.parametrize("name,p,layer", CASES)
def test_mask_matches_oracle_on_every_workload(name, p, layer):
    w = WORKLOADS[name]
    print("mask case", name, p, layer, flush=True)
    m = sdrop.sdrop_mask(w.M, w.K, w.BM, w.BK, p, w.mask_seed, layer)
    _check_mask(m, orc.mask(w.MB, w.KB, p, w.mask_seed, layer))


@pytest.mark.parametrize("M,K,BM,BK,p,seed,stream", [
    (64, 64, 64, 64, 0.5, 1, 0),                 # a single block
    (64, 64, 64, 64, 1.0, 1, 0),
    (128 * 3, 64 * 70, 128, 64, 0.4, 5, 9),      # KB = 70: two mask words per row
    (64 * 1100, 128 * 3, 64, 128, 0.6, 2**40 + 7, 2**33 + 1),   # MB > 1024: several scan chunks; 64-bit seed/stream
    (128 * 5, 128 * 64, 128, 128, 0.0, 3, 3),    # exactly one full word, all kept
    (128 * 5, 128 * 65, 128, 128, 2.0 ** -32, 0, 0),
    (64 * 200, 64 * 130, 64, 64, 0.9, 4, 4),     # sparse, three words per row
    (64 * 2100, 64 * 2, 64, 64, 0.5, 6, 1),      # MB > 2048: the list builder that works in global memory
    (128 * 3, 64 * 2100, 128, 64, 0.25, 7, 2),   # KB > 2048: 33 words per row
    (128 * 64, 128 * 1, 128, 128, 0.5, 8, 0),    # a single block column
    # narrow grids drawn by the list kernel itself, several block rows per wavefront and ballot
    (64 * 7, 64 * 20, 64, 64, 0.5, 9, 0),        # KB = 20 (two rows per ballot), odd number of rows
    (128 * 13, 128 * 5, 128, 128, 0.3, 10, 1),   # KB = 5 (eight rows per ballot), 13 rows
    (64 * 33, 64 * 32, 64, 64, 0.6, 11, 2),      # KB = 32 exactly, 33 rows
    (64 * 50, 64 * 1, 64, 64, 0.5, 12, 3),       # KB = 1: 64 rows per ballot
    (128 * 2, 128 * 17, 128, 128, 0.4, 13, 4),   # KB = 17 rounds up to 32
])
def test_mask_edge_shapes(M, K, BM, BK, p, seed, stream):
    print("mask edge", M, K, BM, BK, p, seed, stream, flush=True)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, stream)
    _check_mask(m, orc.mask(M // BM, K // BK, p, seed, stream))


@pytest.mark.parametrize("M,K,BM,BK,sm,sk,p,seed,stream", [
    (512, 512, 64, 64, 2, 2, 0.5, 1, 0),               # 8 x 8 blocks from a 4 x 4 logical mask (bits drawn by the list kernel)
    (128 * 32, 128 * 32, 128, 128, 2, 1, 0.5, 0, 3),   # logical 256 x 128
    (64 * 96, 64 * 140, 64, 64, 3, 2, 0.3, 5, 1),      # three words per row; factors that are not powers of two
    (64 * 2100, 64 * 4, 64, 64, 2, 4, 0.6, 2, 2),      # more than 2048 block rows: the list builder in global memory
    (128 * 6, 64 * 10, 128, 64, 1, 2, 0.4, 8, 0),      # the forward pass's use in Section 3.3: K-blocks halved
])
def test_block_splitting_matches_oracle(M, K, BM, BK, sm, sk, p, seed, stream):
    print("mask split", M, K, BM, BK, sm, sk, p, seed, stream, flush=True)
    m = sdrop.sdrop_mask_split(M, K, BM, BK, sm, sk, p, seed, stream)
    _check_mask(m, orc.mask_split(M // BM, K // BK, sm, sk, p, seed, stream))


def test_mask_is_reproducible_and_reusable():
    a = sdrop.sdrop_mask(4096, 4096, 128, 128, 0.5, 0, 0)
    b = sdrop.sdrop_mask(4096, 4096, 128, 128, 0.5, 0, 0)
    torch.cuda.synchronize()
    assert torch.equal(a.bits(), b.bits())
    for k in ("row_ptr", "col_idx", "blk_row", "col_ptr", "row_idx", "loc_row", "loc_col"):
        assert torch.equal(a.lists()[k], b.lists()[k])
    # a buffer that held another mask is fully rewritten
    sdrop.sdrop_mask(4096, 4096, 128, 128, 0.1, 7, 1, out=a)
    _check_mask(a, orc.mask(32, 32, 0.1, 7, 1))


def test_mask_from_bits():
    rng = np.random.default_rng(0)
    for (MB, KB, BM, BK) in ((4, 4, 64, 64), (9, 70, 128, 64), (33, 5, 64, 128)):
        keep = (rng.random((MB, KB)) < 0.5).astype(np.uint8)
        words = orc.pack_bits(keep)
        # junk in the unused high bits must be ignored
        if KB % 64:
            words[:, -1] |= np.uint64(0xFFFFFFFFFFFFFFFF) << np.uint64(KB % 64)
        bits = torch.from_numpy(words.view(np.int64)).cuda()
        m = sdrop.sdrop_mask_from_bits(MB * BM, KB * BK, BM, BK, 0.5, bits)
        _check_mask(m, keep)
    none = torch.zeros((4, 1), dtype=torch.int64, device="cuda")
    m = sdrop.sdrop_mask_from_bits(256, 256, 64, 64, 0.5, none)
    _check_mask(m, np.zeros((4, 4), dtype=np.uint8))


def test_mask_bits_reads_the_object_back_through_the_c_abi():
    # sdrop_mask_bits, called raw: host buffers, the one call that waits for the stream
    import ctypes
    L = sdrop.lib()
    vp = ctypes.c_void_p
    for (M, K, BM, BK, p, seed) in ((4096, 4096, 128, 128, 0.5, 0), (576, 64 * 70, 64, 64, 0.3, 5)):
        m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 2)          # enqueued only: the call below must wait for it
        keep = orc.mask(M // BM, K // BK, p, seed, 2)
        want = orc.pack_bits(keep)
        words = np.full(want.shape, 0xDEADBEEF, dtype=np.uint64)
        nnz = ctypes.c_int64(-1)
        rc = L.sdrop_mask_bits(vp(m.buf.data_ptr()), words.ctypes.data_as(vp), words.size, ctypes.byref(nnz), sdrop._stream())
        assert rc == sdrop.OK
        assert np.array_equal(words, want) and nnz.value == int(keep.sum())
        # nnz alone; bits alone
        nnz2 = ctypes.c_int64(-1)
        assert L.sdrop_mask_bits(vp(m.buf.data_ptr()), None, 0, ctypes.byref(nnz2), sdrop._stream()) == sdrop.OK
        assert nnz2.value == nnz.value
        # too few words: refused, the bits untouched
        short = np.full(want.size - 1, 7, dtype=np.uint64)
        assert L.sdrop_mask_bits(vp(m.buf.data_ptr()), short.ctypes.data_as(vp), short.size, None, sdrop._stream()) == sdrop.EWORKSPACE
        assert np.all(short == 7)
        got, n = sdrop.mask_bits_host(m)
        assert np.array_equal(got, want) and n == nnz.value
    # a buffer that holds no mask object
    junk = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    w1 = np.zeros(4, dtype=np.uint64)
    assert L.sdrop_mask_bits(vp(junk.data_ptr()), w1.ctypes.data_as(vp), 4, None, sdrop._stream()) == sdrop.EINVAL
    assert L.sdrop_mask_bits(None, w1.ctypes.data_as(vp), 4, None, None) == sdrop.EINVAL
    assert L.sdrop_mask_bits(vp(junk.data_ptr()), None, 0, None, None) == sdrop.EINVAL


def test_reusing_a_mask_object_for_another_shape_is_refused_by_the_binding():
    m = sdrop.sdrop_mask(512, 512, 128, 128, 0.5, 0, 0)
    with pytest.raises(sdrop.SdropError):
        sdrop.sdrop_mask(512, 512, 64, 64, 0.5, 0, 0, out=m)
    with pytest.raises(sdrop.SdropError):
        sdrop.sdrop_mask_split(1024, 512, 128, 128, 2, 1, 0.5, 0, 0, out=m)
