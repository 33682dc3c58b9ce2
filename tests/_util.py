"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch

# tolerance of the parity gate: relative Frobenius error and max-abs error relative
# to the largest reference magnitude, for fp32-accumulated results
REL_FRO = 1e-3
MAX_ABS = 5e-3
# regression gate for fp32 outputs of eq. (1)-(3): a length-n fp32 sum of exact 16-bit products, added in
# groups of 16, errs by about 2^-24 * sqrt(n / 16) of the result (2e-6 for the longest reduction of the
# workloads, n = 46000; measured 1e-7 to 1e-6).  1e-5 is above all of that and far below what a 16-bit
# accumulation (1e-3), a lost slice of a reduction or a wrong tile would cost.
TIGHT = 1e-5


def f64(t):
    """Exact widening of a 16-bit (or fp32) torch tensor to a float64 numpy array."""
    return t.detach().cpu().to(torch.float64).numpy()


def errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    fro = np.linalg.norm(got - ref) / den if den > 0 else np.linalg.norm(got - ref)
    mx = np.max(np.abs(ref)) if ref.size else 0.0
    mabs = (np.max(np.abs(got - ref)) / mx if mx > 0 else np.max(np.abs(got - ref))) if ref.size else 0.0
    return fro, mabs


def assert_close(got, ref, what, rel_fro=REL_FRO, max_abs=MAX_ABS):
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    fro, mabs = errors(got, ref)
    assert fro <= rel_fro, "%s: relative Frobenius error %.3e > %.1e" % (what, fro, rel_fro)
    assert mabs <= max_abs, "%s: max-abs error %.3e of max|ref| > %.1e" % (what, mabs, max_abs)
    return fro, mabs


def assert_tight(got, ref, what, tol=TIGHT):
    """The regression gate for fp32 outputs (see TIGHT): both error measures at most tol."""
    fro, mabs = errors(got, ref)
    assert fro <= tol and mabs <= tol, "%s: rel-Frobenius %.3e / max-abs %.3e of max|ref| above the regression gate %.0e" % (
        what, fro, mabs, tol)
    return fro, mabs


def bf16_round(a64):
    """Round-to-nearest-even of float64 values to bf16, returned as float64."""
    return torch.from_numpy(np.asarray(a64, dtype=np.float64)).to(torch.bfloat16).to(torch.float64).numpy()


def assert_bf16_rounding_of(got16, ref, what, acc_tol=2e-5):
    """A bf16 output must be the rounding of an accurate fp32 result: each entry within half a
    bf16 ulp of the reference (2^-8 relative, 8 significand bits) plus the fp32 accumulation
    allowance acc_tol * max|ref| (a length-K fp32 sum of exact 16-bit products errs by about
    sqrt(K) * 2^-24 of its partial sums: 4e-6 at K = 4096; the allowance is 5x that)."""
    got16 = np.asarray(got16, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    mx = np.max(np.abs(ref)) if ref.size else 0.0
    bound = np.abs(ref) * (2.0 ** -8) * (1 + 2.0 ** -7) + acc_tol * mx
    bad = np.abs(got16 - ref) > bound
    assert not bad.any(), "%s: %d entries further than half a bf16 ulp + %.0e*max from the oracle" % (
        what, int(bad.sum()), acc_tol)


def lists_from_keep(keep):
    """The index lists a mask object must hold, derived from keep flags with numpy."""
    keep = np.asarray(keep, dtype=np.uint8)
    MB, KB = keep.shape
    row_ptr = np.concatenate([[0], np.cumsum(keep.sum(axis=1))]).astype(np.int32)
    rows, cols = np.nonzero(keep)                      # row-major order
    col_ptr = np.concatenate([[0], np.cumsum(keep.sum(axis=0))]).astype(np.int32)
    crows, ccols = np.nonzero(keep.T)                  # column-major order: (col, row)
    # the same blocks sorted by (row // 8, column, row % 8)
    o = np.lexsort((rows % 8, cols, rows // 8))
    return {"row_ptr": row_ptr, "col_idx": cols.astype(np.int32), "blk_row": rows.astype(np.int32),
            "col_ptr": col_ptr, "row_idx": ccols.astype(np.int32),
            "loc_row": rows[o].astype(np.int32), "loc_col": cols[o].astype(np.int32)}


UNIT_WIDE, UNIT_TALL, UNIT_SINGLE = 0, 1, 2


def units_from_keep(keep):
    """The pair list of a mask object (grids of at most 128 x 64 blocks), by the rule the library documents:
    rows in ascending order; a row with an odd number of kept blocks gives one away, the lowest column in which
    an earlier row's block is still waiting (the two form a tall pair), else its own highest kept column, where
    the block then waits; the rest of the row pairs up left to right; what still waits at the end is single.
    Listed as wide pairs row by row, tall pairs in the order they were closed, singles by column.
    Entries are (kind, x, y, z): wide (i, j1, j2), tall (j, i1, i2), single (i, j, j)."""
    keep = np.asarray(keep, dtype=np.uint8)
    MB, KB = keep.shape
    wide, tall, waiting = [], [], {}
    for i in range(MB):
        cols = [int(j) for j in np.nonzero(keep[i])[0]]
        if len(cols) % 2:
            hits = [j for j in cols if j in waiting]
            if hits:
                c = hits[0]
                tall.append((UNIT_TALL, c, waiting.pop(c), i))
            else:
                c = cols[-1]
                waiting[c] = i
            cols.remove(c)
        wide += [(UNIT_WIDE, i, cols[t], cols[t + 1]) for t in range(0, len(cols), 2)]
    single = [(UNIT_SINGLE, waiting[c], c, c) for c in sorted(waiting)]
    return wide + tall + single


def decode_units(entries):
    return [((int(e) >> 30) & 3, (int(e) >> 16) & 255, (int(e) >> 8) & 255, int(e) & 255) for e in entries]


def blocks_of_units(units):
    """The kept blocks a pair list covers, as a list of (i, j) with repetitions kept."""
    out = []
    for kind, x, y, z in units:
        if kind == UNIT_WIDE:
            out += [(x, y), (x, z)]
        elif kind == UNIT_TALL:
            out += [(y, x), (z, x)]
        else:
            out.append((x, y))
    return out
