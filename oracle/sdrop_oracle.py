"""ctypes front end of the float64 CPU oracle in ``sdrop_oracle.c``.

TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this.  It never touches the HIP library.

Every function takes and returns numpy arrays (float64 matrices, uint8 keep
flags).  The arithmetic lives in the C file; this module only marshals
arguments.  The C file cites the passages of arxiv 2411.01238 it follows
(Section 3.1 eq. (1)-(3), Section 3.2, Section 2.2 footnote).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdrop_oracle.c")
_LIB = os.path.join(_HERE, "libsdrop_oracle.so")

_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain C99 + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_i64 = ctypes.c_int64
_u64 = ctypes.c_uint64
_dbl = ctypes.c_double
_ptr = ctypes.c_void_p


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.sdo_philox4x32_10.argtypes = [_ptr, _ptr, _ptr]
        lib.sdo_philox4x32_10.restype = None
        lib.sdo_block_word.argtypes = [_u64, _u64, _u64]
        lib.sdo_block_word.restype = ctypes.c_uint32
        lib.sdo_threshold.argtypes = [_dbl]
        lib.sdo_threshold.restype = _u64
        lib.sdo_mask_rows.argtypes = [_i64, _i64, _i64, _dbl, _u64, _u64, _ptr]
        lib.sdo_mask_rows.restype = ctypes.c_int
        lib.sdo_pack_bits.argtypes = [_ptr, _i64, _i64, _ptr]
        lib.sdo_pack_bits.restype = ctypes.c_int
        for name in ("sdo_fwd", "sdo_bwd_dx", "sdo_bwd_dw"):
            f = getattr(lib, name)
            f.argtypes = [_ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _i64, _dbl, _ptr]
            f.restype = ctypes.c_int
        for name in ("sdo_fwd_at", "sdo_bwd_dx_at", "sdo_bwd_dw_at"):
            f = getattr(lib, name)
            f.argtypes = [_ptr, _ptr, _ptr, _i64, _i64, _i64, _i64, _i64, _dbl, _i64, _ptr, _ptr, _ptr]
            f.restype = ctypes.c_int
        lib.sdo_threads.argtypes = []
        lib.sdo_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return a.ctypes.data_as(_ptr)


def threads():
    return int(_load().sdo_threads())


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    _load().sdo_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def block_word(seed, stream, b):
    return int(_load().sdo_block_word(seed, stream, b))


def threshold(p):
    return int(_load().sdo_threshold(float(p)))


def mask_rows(i0, i1, KB, p, seed, stream):
    keep = np.zeros((i1 - i0, KB), dtype=np.uint8)
    rc = _load().sdo_mask_rows(i0, i1, KB, float(p), seed, stream, _p(keep))
    if rc != 0:
        raise ValueError("sdo_mask_rows: bad argument")
    return keep


def mask(MB, KB, p, seed, stream):
    """keep[MB, KB] uint8, 1 = block kept (Section 3.2)."""
    return mask_rows(0, MB, KB, p, seed, stream)


def mask_split(MB, KB, split_m, split_k, p, seed, stream):
    """Block splitting (Section 3.3): the logical mask has (MB/split_m) x (KB/split_k) blocks; the
    retiled mask keep[MB, KB] repeats each logical entry split_m times along M and split_k times
    along K.  (The section's text and its figure caption disagree on which of the two factors goes
    with which axis; this follows the text's formula, new block = (Mblk/p, Kblk/q).)"""
    if split_m < 1 or split_k < 1 or MB % split_m or KB % split_k:
        raise ValueError("mask_split: the split factors must divide the block grid")
    logical = mask(MB // split_m, KB // split_k, p, seed, stream)
    return np.repeat(np.repeat(logical, split_m, axis=0), split_k, axis=1)


def pack_bits(keep):
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    MB, KB = keep.shape
    words = np.zeros((MB, (KB + 63) // 64), dtype=np.uint64)
    rc = _load().sdo_pack_bits(_p(keep), MB, KB, _p(words))
    if rc != 0:
        raise ValueError("sdo_pack_bits: bad argument")
    return words


def _gemm(name, A, B, keep, M, K, N, BM, BK, p, out_shape):
    A = _f64(A)
    B = _f64(B)
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    if M % BM or K % BK or keep.shape != (M // BM, K // BK):
        raise ValueError("%s: block sizes must divide the shape and match the mask" % name)
    out = np.empty(out_shape, dtype=np.float64)
    rc = getattr(_load(), name)(_p(A), _p(B), _p(keep), M, K, N, BM, BK, float(p), _p(out))
    if rc != 0:
        raise ValueError("%s: bad argument" % name)
    return out


def fwd(X, W, keep, BM, BK, p):
    """eq. (1): Y = (X . m') W / (1-p)."""
    M, K = X.shape
    K2, N = W.shape
    assert K == K2
    return _gemm("sdo_fwd", X, W, keep, M, K, N, BM, BK, p, (M, N))


def bwd_dx(dY, W, keep, BM, BK, p):
    """eq. (2): dX = (dY W^T) . m' / (1-p)."""
    M, N = dY.shape
    K, N2 = W.shape
    assert N == N2
    return _gemm("sdo_bwd_dx", dY, W, keep, M, K, N, BM, BK, p, (M, K))


def bwd_dw(X, dY, keep, BM, BK, p):
    """eq. (3): dW = (X . m')^T dY / (1-p)."""
    M, K = X.shape
    M2, N = dY.shape
    assert M == M2
    return _gemm("sdo_bwd_dw", X, dY, keep, M, K, N, BM, BK, p, (K, N))


# The same three products for a weight stored as Wt[N,K], one row per output feature (the [out, in] layout
# of common frameworks; Section 3.1 writes W in R^{K x N}, so Wt is its transpose).  Defined through the
# functions above on an explicit transposed copy: W[k][n] = Wt[n][k].
def fwd_wt(X, Wt, keep, BM, BK, p):
    """eq. (1) with W given as Wt[N,K]: Y = (X . m') Wt^T / (1-p)."""
    return fwd(X, np.ascontiguousarray(np.asarray(Wt, dtype=np.float64).T), keep, BM, BK, p)


def bwd_dx_wt(dY, Wt, keep, BM, BK, p):
    """eq. (2) with W given as Wt[N,K]: dX = (dY Wt) . m' / (1-p)."""
    return bwd_dx(dY, np.ascontiguousarray(np.asarray(Wt, dtype=np.float64).T), keep, BM, BK, p)


def bwd_dw_wt(X, dY, keep, BM, BK, p):
    """eq. (3) with the gradient delivered in the weight's [N,K] layout: dWt = dY^T (X . m') / (1-p)."""
    return np.ascontiguousarray(bwd_dw(X, dY, keep, BM, BK, p).T)


def _gemm_at(name, A, B, keep, M, K, N, BM, BK, p, rows, cols):
    A = _f64(A)
    B = _f64(B)
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    if M % BM or K % BK or keep.shape != (M // BM, K // BK):
        raise ValueError("%s: block sizes must divide the shape and match the mask" % name)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    assert rows.shape == cols.shape and rows.ndim == 1
    out = np.empty(rows.shape[0], dtype=np.float64)
    rc = getattr(_load(), name)(_p(A), _p(B), _p(keep), M, K, N, BM, BK, float(p),
                                rows.shape[0], _p(rows), _p(cols), _p(out))
    if rc != 0:
        raise ValueError("%s: bad argument" % name)
    return out


def fwd_at(X, W, keep, BM, BK, p, rows, cols):
    M, K = X.shape
    N = W.shape[1]
    assert np.all((0 <= rows) & (rows < M)) and np.all((0 <= cols) & (cols < N))
    return _gemm_at("sdo_fwd_at", X, W, keep, M, K, N, BM, BK, p, rows, cols)


def bwd_dx_at(dY, W, keep, BM, BK, p, rows, cols):
    M, N = dY.shape
    K = W.shape[0]
    assert np.all((0 <= rows) & (rows < M)) and np.all((0 <= cols) & (cols < K))
    return _gemm_at("sdo_bwd_dx_at", dY, W, keep, M, K, N, BM, BK, p, rows, cols)


def bwd_dw_at(X, dY, keep, BM, BK, p, rows, cols):
    M, K = X.shape
    N = dY.shape[1]
    assert np.all((0 <= rows) & (rows < K)) and np.all((0 <= cols) & (cols < N))
    return _gemm_at("sdo_bwd_dw_at", X, dY, keep, M, K, N, BM, BK, p, rows, cols)
