"""Pins for the oracle's mask rule (CPU only).

The generator core is pinned by the published known-answer vectors; the
counter/key placement by reading those same vectors as (block, stream, seed);
the threshold and keep rule by closed-form cases; the Bernoulli rate
(Section 3.2 of arxiv 2411.01238: one Bernoulli(1-p) per block) by
concentration.
"""
import math
import os

import numpy as np
import pytest

from oracle import sdrop_oracle as orc

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLD, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    assert len(rows) == 3
    return rows


def test_philox_known_answers():
    for ctr, key, want in _kat_rows():
        got = orc.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_block_word_places_counter_and_key_words():
    # the same vectors, read as 64-bit block number / stream / seed; all four
    # counter words and both key words differ in the third vector, so a swapped
    # or dropped word changes the answer
    for ctr, key, want in _kat_rows():
        b = ctr[0] | (ctr[1] << 32)
        stream = ctr[2] | (ctr[3] << 32)
        seed = key[0] | (key[1] << 32)
        assert orc.block_word(seed, stream, b) == want[0]


def test_threshold_closed_forms():
    assert orc.threshold(0.0) == 0
    assert orc.threshold(1.0) == 1 << 32
    assert orc.threshold(0.5) == 1 << 31
    assert orc.threshold(0.25) == 1 << 30
    assert orc.threshold(2.0 ** -32) == 1
    assert orc.threshold(0.1) == math.floor(0.1 * 2 ** 32) == 429496729
    assert orc.threshold(0.7) == 3006477107


def test_keep_rule_is_word_at_least_threshold():
    MB, KB, seed, stream = 6, 10, 7, 3
    for p in (0.0, 0.1, 0.3, 0.5, 0.7, 1.0):
        keep = orc.mask(MB, KB, p, seed, stream)
        T = orc.threshold(p)
        for i in range(MB):
            for j in range(KB):
                r = orc.block_word(seed, stream, i * KB + j)
                assert keep[i, j] == (1 if r >= T else 0)


def test_p0_keeps_all_p1_drops_all():
    assert orc.mask(5, 7, 0.0, 11, 2).all()
    assert not orc.mask(5, 7, 1.0, 11, 2).any()


def test_smallest_p_drops_only_word_zero():
    # with T = 1 a block is dropped only if its word is exactly 0
    keep = orc.mask(64, 64, 2.0 ** -32, 0, 0)
    words = np.array([[orc.block_word(0, 0, i * 64 + j) for j in range(64)] for i in range(64)])
    assert np.array_equal(keep == 0, words == 0)


def test_kept_sets_are_nested_in_p():
    prev = orc.mask(16, 16, 0.0, 5, 5)
    for p in (0.1, 0.3, 0.5, 0.7, 0.9, 1.0):
        cur = orc.mask(16, 16, p, 5, 5)
        assert np.all(cur <= prev)
        prev = cur


def test_row_range_is_slice_of_whole_mask():
    MB, KB = 37, 13
    whole = orc.mask(MB, KB, 0.4, 9, 1)
    for i0, i1 in ((0, 5), (5, 20), (20, 37), (36, 37), (7, 7)):
        part = orc.mask_rows(i0, i1, KB, 0.4, 9, 1)
        assert np.array_equal(part, whole[i0:i1])


def test_seed_and_stream_change_the_mask():
    a = orc.mask(32, 32, 0.5, 0, 0)
    assert not np.array_equal(a, orc.mask(32, 32, 0.5, 1, 0))
    assert not np.array_equal(a, orc.mask(32, 32, 0.5, 0, 1))
    assert not np.array_equal(orc.mask(32, 32, 0.5, 1, 0), orc.mask(32, 32, 0.5, 0, 1))
    assert np.array_equal(a, orc.mask(32, 32, 0.5, 0, 0))


@pytest.mark.parametrize("MB,KB,p", [(32, 32, 0.5), (32, 32, 0.1), (512, 32, 0.3),
                                       (128, 48, 0.1), (128, 16, 0.5), (32, 32, 0.7)])
def test_kept_fraction_concentrates_at_one_minus_p(MB, KB, p):
    keep = orc.mask(MB, KB, p, 0, 0)
    n = MB * KB
    assert abs(keep.mean() - (1.0 - p)) <= 4.0 * math.sqrt(p * (1.0 - p) / n)


def test_kept_fraction_over_streams_tiny():
    # 64 independent streams of the 4x4 grid: 1024 draws
    tot = sum(int(orc.mask(4, 4, 0.5, 0, s).sum()) for s in range(64))
    assert abs(tot / 1024.0 - 0.5) <= 4.0 * math.sqrt(0.25 / 1024)


def test_rows_and_columns_are_not_correlated():
    # a transposed block index (j*MB+i instead of i*KB+j) would pass the rate
    # test; it fails here because the grid is not square
    a = orc.mask(3, 5, 0.5, 2, 0)
    flat = np.array([1 if orc.block_word(2, 0, b) >= (1 << 31) else 0 for b in range(15)])
    assert np.array_equal(a.reshape(-1), flat)


def test_pack_bits_layout():
    keep = np.zeros((2, 70), dtype=np.uint8)
    keep[0, 0] = 1
    keep[0, 63] = 1
    keep[0, 64] = 1
    keep[1, 1] = 1
    keep[1, 69] = 1
    w = orc.pack_bits(keep)
    assert w.shape == (2, 2)
    assert int(w[0, 0]) == (1 | (1 << 63))
    assert int(w[0, 1]) == 1
    assert int(w[1, 0]) == 2
    assert int(w[1, 1]) == 1 << 5


def test_tiny_workload_fixture():
    vals = {}
    with open(os.path.join(GOLD, "mask_tiny_seed0.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            k, *rest = line.split()
            vals[k] = rest
    words = [int(x) for x in vals["words"]]
    assert [orc.block_word(0, 0, b) for b in range(16)] == words
    # block 0 of seed 0 / stream 0 is the first published known-answer word
    assert words[0] == 0x6627E8D5
    keep = orc.mask(4, 4, 0.5, 0, 0)
    assert [int(v) for v in keep.reshape(-1)] == [int(x) for x in vals["keep"]]
    assert [int(v) for v in orc.pack_bits(keep).reshape(-1)] == [int(x, 16) for x in vals["packed"]]
    assert int(keep.sum()) == 10


def _elementwise(keep, BM, BK):
    return np.repeat(np.repeat(keep, BM, axis=0), BK, axis=1)


def test_block_splitting_keeps_the_semantics_of_the_logical_mask():
    # Section 3.3, Figure 3: a logical mask with 2x2-element blocks, the same mask retiled to 2x1- or
    # 1x2-element blocks ("operates on" half blocks), and to 1x1, mask exactly the same elements
    seed, stream, p = 9, 4, 0.5
    logical = orc.mask(3, 5, p, seed, stream)
    assert 0 < logical.sum() < 15
    want = _elementwise(logical, 2, 2)
    for sm, sk in ((1, 1), (2, 1), (1, 2), (2, 2)):
        split = orc.mask_split(3 * sm, 5 * sk, sm, sk, p, seed, stream)
        assert split.shape == (3 * sm, 5 * sk)
        assert np.array_equal(_elementwise(split, 2 // sm, 2 // sk), want), (sm, sk)
    assert np.array_equal(orc.mask_split(3, 5, 1, 1, p, seed, stream), logical)


def test_block_splitting_entry_by_entry_and_axes():
    # entry (i, j) of the retiled mask is the keep decision of logical block (i // split_m, j // split_k),
    # numbered row-major over the LOGICAL grid; a non-square case tells the two axes apart
    seed, stream, p, sm, sk = 3, 1, 0.4, 3, 2
    MBL, KBL = 4, 7
    split = orc.mask_split(MBL * sm, KBL * sk, sm, sk, p, seed, stream)
    thr = orc.threshold(p)
    for i in range(MBL * sm):
        for j in range(KBL * sk):
            b = (i // sm) * KBL + (j // sk)
            assert split[i, j] == (1 if orc.block_word(seed, stream, b) >= thr else 0)
    # rows repeat in runs of split_m, columns in runs of split_k
    assert all(np.array_equal(split[i], split[i - i % sm]) for i in range(MBL * sm))
    assert all(np.array_equal(split[:, j], split[:, j - j % sk]) for j in range(KBL * sk))
    with pytest.raises(ValueError):
        orc.mask_split(7, 8, 2, 2, p, seed, stream)
