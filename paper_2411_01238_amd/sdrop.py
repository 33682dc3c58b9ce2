"""Thin ctypes binding over libsdrop.so (the C ABI declared in include/sdrop.h).

Argument marshalling only: every function below passes device pointers of torch
tensors, sizes and the current HIP stream straight to the C entry point of the
same name.  There is no CPU fallback: if the library is not built, or a call is
made without a GPU tensor, it raises.

The operations are those of arxiv 2411.01238, Section 3.1 eq. (1)-(3) with the
block mask of Section 3.2; see the header for the full contract.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdrop.so")

OK, EINVAL, ESHAPE, EDTYPE, EALIGN, EWORKSPACE, EHIP = range(7)
F16, BF16, F32 = 0, 1, 2
OP_FWD, OP_BWD_DX, OP_BWD_DW = 0, 1, 2
MASK_NNZ_OFFSET = 36
MASK_NUNITS_OFFSET = 80

EXPORTS = ("sdrop_strerror", "sdrop_last_hip_error", "sdrop_status", "sdrop_set_tuning", "sdrop_mask_layout", "sdrop_mask_bytes",
           "sdrop_mask", "sdrop_mask_split", "sdrop_mask_from_bits", "sdrop_mask_bits", "sdrop_workspace_bytes",
           "sdrop_fwd", "sdrop_fwd_seeded", "sdrop_fwd_seeded_ex", "sdrop_bwd_dx", "sdrop_bwd_dw", "sdrop_bwd_dw_static",
           "sdrop_bwd", "sdrop_bwd_ex", "sdrop_fwd_ex", "sdrop_bwd_dx_ex", "sdrop_bwd_dw_ex", "sdrop_workspace_bytes_ex",
           "sdrop_producer", "sdrop_producer_ex",
           "sdrop_bias_grad_workspace_bytes", "sdrop_bias_grad")

SCALE_DROPOUT, SCALE_ONE = 0, 1
ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_GELU_ERF = 0, 1, 2, 3
GATE_RELU, GATE_GELU_TANH, GATE_GELU_ERF = 0, 1, 2
W_KN, W_NK = 0, 1

_DTYPES = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}


class SdropError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %s (code %d)" % (what, strerror(code), code))


class MaskLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in
                ("total_bytes", "off_bits", "off_row_ptr", "off_col_idx", "off_blk_row",
                 "off_col_ptr", "off_row_idx", "off_row_order", "off_col_order", "off_loc_row", "off_loc_col", "off_units")] + \
               [(n, ctypes.c_int64) for n in ("MB", "KB", "words_per_row")]


class Epilogue(ctypes.Structure):
    """sdrop_epilogue_t of the header."""
    _fields_ = [("scale_mode", ctypes.c_int32), ("act", ctypes.c_int32),
                ("bias", ctypes.c_void_p), ("relu_mask", ctypes.c_void_p),
                ("ld_a", ctypes.c_int64), ("ld_b", ctypes.c_int64), ("ld_out", ctypes.c_int64),
                ("gate_mode", ctypes.c_int32), ("w_layout", ctypes.c_int32), ("kept_fraction", ctypes.c_double)]


_lib = None


def lib():
    """Loads libsdrop.so; raises if it has not been built (python -m paper_2411_01238_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsdrop.so is not built: run `python -m paper_2411_01238_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        i64, u64, dbl, vp, ci, sz = (ctypes.c_int64, ctypes.c_uint64, ctypes.c_double,
                                     ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t)
        L.sdrop_strerror.argtypes = [ci]
        L.sdrop_strerror.restype = ctypes.c_char_p
        L.sdrop_last_hip_error.argtypes = []
        L.sdrop_last_hip_error.restype = ci
        L.sdrop_status.argtypes = [ctypes.POINTER(ci), ci, vp]
        L.sdrop_status.restype = ci
        L.sdrop_set_tuning.argtypes = [ci, ci]
        L.sdrop_set_tuning.restype = ci
        L.sdrop_mask_layout.argtypes = [i64, i64, ci, ci, ctypes.POINTER(MaskLayout)]
        L.sdrop_mask_layout.restype = ci
        L.sdrop_mask_bytes.argtypes = [i64, i64, ci, ci]
        L.sdrop_mask_bytes.restype = sz
        L.sdrop_mask.argtypes = [vp, sz, i64, i64, ci, ci, dbl, u64, u64, vp]
        L.sdrop_mask.restype = ci
        L.sdrop_mask_split.argtypes = [vp, sz, i64, i64, ci, ci, ci, ci, dbl, u64, u64, vp]
        L.sdrop_mask_split.restype = ci
        L.sdrop_mask_from_bits.argtypes = [vp, sz, i64, i64, ci, ci, vp, vp]
        L.sdrop_mask_from_bits.restype = ci
        L.sdrop_mask_bits.argtypes = [vp, vp, sz, vp, vp]
        L.sdrop_mask_bits.restype = ci
        L.sdrop_workspace_bytes.argtypes = [ci, i64, i64, i64, ci, ci, ci, ci]
        L.sdrop_workspace_bytes.restype = sz
        for name in ("sdrop_fwd", "sdrop_bwd_dx", "sdrop_bwd_dw"):
            f = getattr(L, name)
            f.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, vp, sz, vp]
            f.restype = ci
        L.sdrop_fwd_seeded.argtypes = [vp, vp, vp, sz, vp, i64, i64, i64, ci, ci, dbl, u64, u64, ci, ci, vp]
        L.sdrop_fwd_seeded.restype = ci
        L.sdrop_fwd_seeded_ex.argtypes = [vp, vp, vp, sz, vp, i64, i64, i64, ci, ci, dbl, u64, u64, ci, ci, vp, sz, vp,
                                          ctypes.POINTER(Epilogue)]
        L.sdrop_fwd_seeded_ex.restype = ci
        L.sdrop_bwd_dw_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, vp]
        L.sdrop_bwd_dw_static.restype = ci
        for name in ("sdrop_fwd_ex", "sdrop_bwd_dx_ex", "sdrop_bwd_dw_ex"):
            f = getattr(L, name)
            f.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, vp, sz, vp, ctypes.POINTER(Epilogue)]
            f.restype = ci
        L.sdrop_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, vp, sz, vp]
        L.sdrop_bwd.restype = ci
        L.sdrop_bwd_ex.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, vp, sz, vp, i64, i64, i64, i64, i64, ci]
        L.sdrop_bwd_ex.restype = ci
        L.sdrop_workspace_bytes_ex.argtypes = [ci, i64, i64, i64, ci, ci, ci, ci, ctypes.POINTER(Epilogue)]
        L.sdrop_workspace_bytes_ex.restype = sz
        L.sdrop_producer_ex.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, ci, vp, i64, i64, i64]
        L.sdrop_producer_ex.restype = ci
        L.sdrop_producer.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, dbl, ci, ci, ci, vp]
        L.sdrop_producer.restype = ci
        L.sdrop_bias_grad_workspace_bytes.argtypes = [i64, i64, ci, ci]
        L.sdrop_bias_grad_workspace_bytes.restype = sz
        L.sdrop_bias_grad.argtypes = [vp, vp, vp, i64, i64, ci, ci, ci, i64, vp, sz, vp]
        L.sdrop_bias_grad.restype = ci
        _lib = L
    return _lib


TUNE_DX_PERSISTENT_GROUPS_PER_CU = 0
DX_PERSISTENT_GROUPS_PER_CU_DEFAULT = 8
TUNE_BWD_FUSED = 1
TUNE_DX_TILE_WIDTH = 2
TUNE_FWD_SEEDED = 3
TUNE_DW64_PERSISTENT_SLICES = 4
TUNE_DX_PAIRS = 5


def set_tuning(knob, value):
    _check(lib().sdrop_set_tuning(int(knob), int(value)), "sdrop_set_tuning")


STATUS_MASK_MISMATCH = 1


def status(clear=True):
    """The library's device-side status word on the current GPU (see sdrop_status): waits for the current stream."""
    v = ctypes.c_int(0)
    _check(lib().sdrop_status(ctypes.byref(v), 1 if clear else 0, _stream()), "sdrop_status")
    return int(v.value)


def strerror(code):
    return lib().sdrop_strerror(int(code)).decode()


def _check(code, what):
    if code != OK:
        raise SdropError(code, what)


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream():
    """The current HIP stream of the current device, as a pointer."""
    if _raw_stream is not None:
        # one C call instead of building a torch.cuda.Stream object (a third of a call's host time)
        return ctypes.c_void_p(_raw_stream(torch.cuda.current_device()))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError("%s must be a contiguous GPU tensor" % name)
    return ctypes.c_void_p(t.data_ptr())


def _mat(t, name):
    """Device pointer and leading dimension (elements) of a 2-D GPU tensor whose rows are contiguous:
    a contiguous matrix or a column range of a wider one."""
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dim() == 2 and (t.shape[1] == 1 or t.stride(1) == 1)
            and (t.shape[0] == 1 or t.stride(0) >= t.shape[1])):
        raise ValueError("%s must be a 2-D GPU tensor with contiguous rows" % name)
    ld = t.stride(0) if t.shape[0] > 1 else t.shape[1]
    return ctypes.c_void_p(t.data_ptr()), int(ld)


def mask_layout(M, K, BM, BK):
    out = MaskLayout()
    _check(lib().sdrop_mask_layout(M, K, BM, BK, ctypes.byref(out)), "sdrop_mask_layout")
    return out


def mask_bytes(M, K, BM, BK):
    return int(lib().sdrop_mask_bytes(M, K, BM, BK))


class Mask:
    """A mask object in device memory (a caller-owned uint8 tensor) plus its shape."""

    def __init__(self, M, K, BM, BK, p, device="cuda"):
        self.M, self.K, self.BM, self.BK, self.p = M, K, BM, BK, float(p)
        self.layout = mask_layout(M, K, BM, BK)
        self.buf = torch.empty(self.layout.total_bytes, dtype=torch.uint8, device=device)

    @property
    def MB(self):
        return int(self.layout.MB)

    @property
    def KB(self):
        return int(self.layout.KB)

    # views for tests and diagnostics (each .cpu() call synchronises)
    def _i32(self, off, n):
        return self.buf[off:off + 4 * n].view(torch.int32)

    def nnz(self):
        return int(self.buf[MASK_NNZ_OFFSET:MASK_NNZ_OFFSET + 4].view(torch.int32).item())

    def n_units(self):
        """Entries of the pair list (0 for grids it is not built for)."""
        return int(self.buf[MASK_NUNITS_OFFSET:MASK_NUNITS_OFFSET + 4].view(torch.int32).item())

    def bits(self):
        L = self.layout
        n = self.MB * int(L.words_per_row)
        return self.buf[L.off_bits:L.off_bits + 8 * n].view(torch.int64).reshape(self.MB, -1)

    def lists(self):
        L = self.layout
        nnz = self.nnz()
        return {
            "row_ptr": self._i32(L.off_row_ptr, self.MB + 1),
            "col_idx": self._i32(L.off_col_idx, nnz),
            "blk_row": self._i32(L.off_blk_row, nnz),
            "col_ptr": self._i32(L.off_col_ptr, self.KB + 1),
            "row_idx": self._i32(L.off_row_idx, nnz),
            "row_order": self._i32(L.off_row_order, self.MB),
            "col_order": self._i32(L.off_col_order, self.KB),
            "loc_row": self._i32(L.off_loc_row, nnz),
            "loc_col": self._i32(L.off_loc_col, nnz),
            "units": self._i32(L.off_units, self.n_units()),
        }


def _mask_out(out, M, K, BM, BK, p):
    """A new Mask, or `out` after checking that it was made for this shape (a reused object's buffer
    and Python fields must agree with what the library is about to write into it)."""
    if out is None:
        return Mask(M, K, BM, BK, p)
    if (out.M, out.K, out.BM, out.BK) != (M, K, BM, BK):
        raise SdropError(ESHAPE, "mask object passed as out= was made for another shape")
    return out


def mask_bits_host(mask):
    """(keep bits as a numpy uint64 array [MB, words_per_row], nnz) of a Mask, through sdrop_mask_bits
    (synchronises with the current stream)."""
    import numpy as np
    words = np.zeros((mask.MB, int(mask.layout.words_per_row)), dtype=np.uint64)
    nnz = ctypes.c_int64(-1)
    _check(lib().sdrop_mask_bits(_dev(mask.buf, "mask"), words.ctypes.data_as(ctypes.c_void_p), words.size,
                                 ctypes.byref(nnz), _stream()), "sdrop_mask_bits")
    return words, int(nnz.value)


def sdrop_mask(M, K, BM, BK, p, seed, rng_stream=0, out=None):
    """Draws the block mask of Section 3.2 on the device; returns a Mask."""
    m = _mask_out(out, M, K, BM, BK, p)
    m.p = float(p)
    _check(lib().sdrop_mask(_dev(m.buf, "mask"), m.buf.numel(), M, K, BM, BK, float(p),
                            int(seed), int(rng_stream), _stream()), "sdrop_mask")
    return m


def sdrop_mask_split(M, K, BM, BK, split_m, split_k, p, seed, rng_stream=0, out=None):
    """Block splitting (Section 3.3): logical blocks of (split_m BM) x (split_k BK), retiled to BM x BK."""
    m = _mask_out(out, M, K, BM, BK, p)
    m.p = float(p)
    _check(lib().sdrop_mask_split(_dev(m.buf, "mask"), m.buf.numel(), M, K, BM, BK, int(split_m), int(split_k),
                                  float(p), int(seed), int(rng_stream), _stream()), "sdrop_mask_split")
    return m


def sdrop_mask_from_bits(M, K, BM, BK, p, bits, out=None):
    """Mask object from given keep bits: int64/uint64 GPU tensor [MB, words_per_row]."""
    m = _mask_out(out, M, K, BM, BK, p)
    m.p = float(p)
    _check(lib().sdrop_mask_from_bits(_dev(m.buf, "mask"), m.buf.numel(), M, K, BM, BK,
                                      _dev(bits, "bits"), _stream()), "sdrop_mask_from_bits")
    return m


_ws_cache = {}


def workspace_bytes(op, M, K, N, BM, BK, dtype, out_dtype):
    key = (op, M, K, N, BM, BK, dtype, out_dtype)
    v = _ws_cache.get(key)
    if v is None:
        v = int(lib().sdrop_workspace_bytes(op, M, K, N, BM, BK, _DTYPES[dtype], _DTYPES[out_dtype]))
        _ws_cache[key] = v
    return v


def _epilogue(scale_mode, act, bias, relu_mask, ncols, out_shape, dtype, gate_mode=GATE_RELU, w_layout=W_KN, kept_fraction=0.0):
    """Marshals the tail arguments into the C struct (leading dimensions are filled in by _gemm)."""
    e = Epilogue()
    e.scale_mode, e.act, e.gate_mode, e.w_layout = int(scale_mode), int(act), int(gate_mode), int(w_layout)
    e.kept_fraction = float(kept_fraction)
    e.bias = e.relu_mask = None
    e.ld_a = e.ld_b = e.ld_out = 0
    if bias is not None:
        if bias.dtype != torch.float32 or tuple(bias.shape) != (ncols,):
            raise ValueError("bias must be fp32 with one value per output column")
        e.bias = _dev(bias, "bias").value
    if relu_mask is not None:
        if relu_mask.dtype != dtype or tuple(relu_mask.shape) != tuple(out_shape):
            raise ValueError("relu_mask must have the operands' dtype and the output's shape")
        ptr, e.relu_mask_ld = _mat(relu_mask, "relu_mask")
        e.relu_mask = ptr.value
    return e


def _gemm(name, op, a, b, mask, out_shape, M, K, N, out_dtype, out, ws, epi=None):
    dtype = a.dtype
    if b.dtype != dtype:
        raise ValueError("operands must have the same dtype")
    out_dtype = dtype if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty(out_shape, dtype=out_dtype, device=a.device)
    elif tuple(out.shape) != tuple(out_shape) or out.dtype != out_dtype:
        raise ValueError("out has the wrong shape or dtype")
    if dtype not in (torch.float16, torch.bfloat16) or out_dtype not in _DTYPES:
        raise SdropError(EDTYPE, name)
    if epi is not None and epi.w_layout != W_KN:
        need = int(lib().sdrop_workspace_bytes_ex(op, M, K, N, mask.BM, mask.BK, _DTYPES[dtype], _DTYPES[out_dtype], ctypes.byref(epi)))
    else:
        need = workspace_bytes(op, M, K, N, mask.BM, mask.BK, dtype, out_dtype)
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=a.device)
    ws_ptr = ctypes.c_void_p(ws.data_ptr()) if ws is not None else ctypes.c_void_p(0)
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    (pa, lda), (pb, ldb), (po, ldo) = _mat(a, "a"), _mat(b, "b"), _mat(out, "out")
    args = (pa, pb, _dev(mask.buf, "mask"), po,
            M, K, N, mask.BM, mask.BK, mask.p, _DTYPES[dtype], _DTYPES[out_dtype], ws_ptr, ws_bytes, _stream())
    strided = (lda, ldb, ldo) != (a.shape[1], b.shape[1], out.shape[1])
    if epi is not None and getattr(epi, "relu_mask_ld", ldo) != ldo:
        raise ValueError("relu_mask must have the output's leading dimension")
    if name.endswith("_ex") or strided:
        # row-strided operands go through the _ex entry point of the same operation
        if epi is None:
            epi = _epilogue(SCALE_DROPOUT, ACT_NONE, None, None, 0, out_shape, dtype)
        if strided:
            epi.ld_a, epi.ld_b, epi.ld_out = lda, ldb, ldo
        ex = name if name.endswith("_ex") else name + "_ex"
        rc = getattr(lib(), ex)(*args, ctypes.byref(epi))
    else:
        rc = getattr(lib(), name)(*args)
    _check(rc, name)
    return out


def sdrop_fwd(X, W, mask, out_dtype=None, out=None, ws=None):
    """eq. (1): Y = s (X . m') W."""
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_fwd")
    return _gemm("sdrop_fwd", OP_FWD, X, W, mask, (M, N), M, K, N, out_dtype, out, ws)


def sdrop_fwd_seeded(X, W, BM, BK, p, seed, rng_stream=0, mask=None, out_dtype=None, out=None, w_layout=W_KN, ws=None):
    """The step's mask and eq. (1) in one call (one launch for small block grids): returns (Y, Mask).
    The Mask is the object sdrop_mask would have written; the backward calls of the step take it.
    w_layout=W_NK: W is given as [N, K].  Row-strided X, W or out (column ranges of wider matrices) are taken in place."""
    M, K = X.shape
    K2, N = W.shape if w_layout == W_KN else (W.shape[1], W.shape[0])
    if K2 != K:
        raise SdropError(ESHAPE, "sdrop_fwd_seeded")
    dtype = X.dtype
    if W.dtype != dtype:
        raise ValueError("operands must have the same dtype")
    out_dtype = dtype if out_dtype is None else out_dtype
    if dtype not in (torch.float16, torch.bfloat16) or out_dtype not in _DTYPES:
        raise SdropError(EDTYPE, "sdrop_fwd_seeded")
    m = _mask_out(mask, M, K, BM, BK, p)
    m.p = float(p)
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=X.device)
    elif tuple(out.shape) != (M, N) or out.dtype != out_dtype:
        raise ValueError("out has the wrong shape or dtype")
    (xp, ldx), (wp, ldw), (yp, ldy) = _mat(X, "X"), _mat(W, "W"), _mat(out, "Y")
    if w_layout == W_KN and (ldx, ldw, ldy) == (K, N, N):
        rc = lib().sdrop_fwd_seeded(xp, wp, _dev(m.buf, "mask"), m.buf.numel(), yp,
                                    M, K, N, BM, BK, float(p), int(seed), int(rng_stream),
                                    _DTYPES[dtype], _DTYPES[out_dtype], _stream())
    else:
        e = _epilogue(SCALE_DROPOUT, ACT_NONE, None, None, N, (M, N), dtype, w_layout=w_layout)
        e.ld_a, e.ld_b, e.ld_out = ldx, ldw, ldy
        need = int(lib().sdrop_workspace_bytes_ex(OP_FWD, M, K, N, BM, BK, _DTYPES[dtype], _DTYPES[out_dtype], ctypes.byref(e)))
        if ws is None and need:
            ws = torch.empty(need, dtype=torch.uint8, device=X.device)
        ws_ptr = ctypes.c_void_p(ws.data_ptr()) if ws is not None else ctypes.c_void_p(0)
        ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
        rc = lib().sdrop_fwd_seeded_ex(xp, wp, _dev(m.buf, "mask"), m.buf.numel(), yp,
                                       M, K, N, BM, BK, float(p), int(seed), int(rng_stream),
                                       _DTYPES[dtype], _DTYPES[out_dtype], ws_ptr, ws_bytes, _stream(), ctypes.byref(e))
    _check(rc, "sdrop_fwd_seeded")
    return out, m


def sdrop_bwd_dx(dY, W, mask, out_dtype=None, out=None, ws=None):
    """eq. (2): dX = s (dY W^T) . m'."""
    M, N = dY.shape
    K, N2 = W.shape
    if N2 != N or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bwd_dx")
    return _gemm("sdrop_bwd_dx", OP_BWD_DX, dY, W, mask, (M, K), M, K, N, out_dtype, out, ws)


def sdrop_bwd_dw(X, dY, mask, out_dtype=None, out=None, ws=None):
    """eq. (3): dW = s (X . m')^T dY."""
    M, K = X.shape
    M2, N = dY.shape
    if M2 != M or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bwd_dw")
    return _gemm("sdrop_bwd_dw", OP_BWD_DW, X, dY, mask, (K, N), M, K, N, out_dtype, out, ws)


STATIC_SCRATCH_BYTES = 128 << 20


def sdrop_bwd_dw_static(X, dY, mask, out, out_dtype=None):
    """eq. (3) through the entry point that allocates nothing: the caller passes the output, the planes of a
    split reduction live in the library's own device memory (at most STATIC_SCRATCH_BYTES)."""
    M, K = X.shape
    M2, N = dY.shape
    if M2 != M or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bwd_dw_static")
    dtype = X.dtype
    out_dtype = dtype if out_dtype is None else out_dtype
    if dY.dtype != dtype or tuple(out.shape) != (K, N) or out.dtype != out_dtype:
        raise ValueError("operands / output have the wrong shape or dtype")
    if dtype not in (torch.float16, torch.bfloat16) or out_dtype not in _DTYPES:
        raise SdropError(EDTYPE, "sdrop_bwd_dw_static")
    rc = lib().sdrop_bwd_dw_static(_dev(X, "X"), _dev(dY, "dY"), _dev(mask.buf, "mask"), _dev(out, "dW"),
                                   M, K, N, mask.BM, mask.BK, mask.p, _DTYPES[dtype], _DTYPES[out_dtype], _stream())
    _check(rc, "sdrop_bwd_dw_static")
    return out


def sdrop_bwd(dY, W, X, mask, out_dtype=None, out_dx=None, out_dw=None, ws=None, w_layout=W_KN):
    """eq. (2) and eq. (3) in one call (one launch where the shapes allow it): returns (dX, dW).
    w_layout=W_NK: W is given, and dW returned, as [N, K]."""
    M, N = dY.shape
    K, N2 = W.shape if w_layout == W_KN else (W.shape[1], W.shape[0])
    if N2 != N or tuple(X.shape) != (M, K) or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bwd")
    dtype = dY.dtype
    if W.dtype != dtype or X.dtype != dtype:
        raise ValueError("operands must have the same dtype")
    out_dtype = dtype if out_dtype is None else out_dtype
    if dtype not in (torch.float16, torch.bfloat16) or out_dtype not in _DTYPES:
        raise SdropError(EDTYPE, "sdrop_bwd")
    outs = []
    for o, shape in ((out_dx, (M, K)), (out_dw, (K, N) if w_layout == W_KN else (N, K))):
        if o is None:
            o = torch.empty(shape, dtype=out_dtype, device=dY.device)
        elif tuple(o.shape) != shape or o.dtype != out_dtype:
            raise ValueError("an output has the wrong shape or dtype")
        outs.append(o)
    if w_layout == W_KN:
        need = workspace_bytes(OP_BWD_DW, M, K, N, mask.BM, mask.BK, dtype, out_dtype)
    else:
        e = _epilogue(SCALE_DROPOUT, ACT_NONE, None, None, N, (K, N), dtype, w_layout=w_layout)
        need = int(lib().sdrop_workspace_bytes_ex(OP_BWD_DW, M, K, N, mask.BM, mask.BK, _DTYPES[dtype], _DTYPES[out_dtype], ctypes.byref(e)))
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=dY.device)
    ws_ptr = ctypes.c_void_p(ws.data_ptr()) if ws is not None else ctypes.c_void_p(0)
    ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    mats = [_mat(t, n) for t, n in ((dY, "dY"), (W, "W"), (X, "X"), (outs[0], "dX"), (outs[1], "dW"))]
    ptrs = [m[0] for m in mats]
    lds = [m[1] for m in mats]
    if w_layout == W_KN and lds == [N, N, K, K, N]:
        rc = lib().sdrop_bwd(ptrs[0], ptrs[1], ptrs[2], _dev(mask.buf, "mask"), ptrs[3], ptrs[4], M, K, N, mask.BM, mask.BK, mask.p,
                             _DTYPES[dtype], _DTYPES[out_dtype], ws_ptr, ws_bytes, _stream())
    else:
        # row-strided operands or outputs (column ranges of wider matrices)
        rc = lib().sdrop_bwd_ex(ptrs[0], ptrs[1], ptrs[2], _dev(mask.buf, "mask"), ptrs[3], ptrs[4], M, K, N, mask.BM, mask.BK, mask.p,
                                _DTYPES[dtype], _DTYPES[out_dtype], ws_ptr, ws_bytes, _stream(), *lds, int(w_layout))
    _check(rc, "sdrop_bwd")
    return outs[0], outs[1]


def sdrop_fwd_ex(X, W, mask, scale_mode=SCALE_DROPOUT, act=ACT_NONE, bias=None, relu_mask=None,
                 out_dtype=None, out=None, ws=None, gate_mode=GATE_RELU, w_layout=W_KN, kept_fraction=0.0):
    """eq. (1) with an element-wise tail: Y = [relu_mask > 0] act(scale (X . m') W + bias).
    w_layout=W_NK: W is given as [N, K] (one row per output feature)."""
    M, K = X.shape
    K2, N = W.shape if w_layout == W_KN else (W.shape[1], W.shape[0])
    if K2 != K or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_fwd_ex")
    epi = _epilogue(scale_mode, act, bias, relu_mask, N, (M, N), X.dtype, gate_mode, w_layout, kept_fraction)
    return _gemm("sdrop_fwd_ex", OP_FWD, X, W, mask, (M, N), M, K, N, out_dtype, out, ws, epi)


def sdrop_bwd_dx_ex(dY, W, mask, scale_mode=SCALE_DROPOUT, act=ACT_NONE, bias=None, relu_mask=None,
                    out_dtype=None, out=None, ws=None, gate_mode=GATE_RELU, w_layout=W_KN, kept_fraction=0.0):
    """eq. (2) with an element-wise tail on the kept blocks; dropped blocks are +0.
    w_layout=W_NK: W is given as [N, K]."""
    M, N = dY.shape
    K, N2 = W.shape if w_layout == W_KN else (W.shape[1], W.shape[0])
    if N2 != N or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bwd_dx_ex")
    epi = _epilogue(scale_mode, act, bias, relu_mask, K, (M, K), dY.dtype, gate_mode, w_layout, kept_fraction)
    return _gemm("sdrop_bwd_dx_ex", OP_BWD_DX, dY, W, mask, (M, K), M, K, N, out_dtype, out, ws, epi)


def sdrop_bwd_dw_ex(X, dY, mask, scale_mode=SCALE_DROPOUT, out_dtype=None, out=None, ws=None, w_layout=W_KN, kept_fraction=0.0):
    """eq. (3) with the scale chosen by scale_mode.  w_layout=W_NK: the gradient comes as [N, K]."""
    M, K = X.shape
    M2, N = dY.shape
    if M2 != M or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bwd_dw_ex")
    out_shape = (K, N) if w_layout == W_KN else (N, K)
    epi = _epilogue(scale_mode, ACT_NONE, None, None, N, out_shape, X.dtype, w_layout=w_layout, kept_fraction=kept_fraction)
    return _gemm("sdrop_bwd_dw_ex", OP_BWD_DW, X, dY, mask, out_shape, M, K, N, out_dtype, out, ws, epi)


def sdrop_producer(H, W0, bias, mask, act=ACT_NONE, out_dtype=None, out=None, preact=None):
    """The layer before the dropout, output-sparse: X = m' . act(H W0^T + bias), W0 is [K, N0].

    preact: None, or a tensor of X's shape and type that receives H W0^T + bias on the kept blocks
    (its dropped blocks are left as they are); True allocates one (zero-filled).  With it the call
    returns (X, preact)."""
    M, N0 = H.shape
    K, N02 = W0.shape
    if N02 != N0 or (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_producer")
    dtype = H.dtype
    if W0.dtype != dtype:
        raise ValueError("operands must have the same dtype")
    out_dtype = dtype if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty((M, K), dtype=out_dtype, device=H.device)
    elif tuple(out.shape) != (M, K) or out.dtype != out_dtype:
        raise ValueError("out has the wrong shape or dtype")
    if dtype not in (torch.float16, torch.bfloat16) or out_dtype not in _DTYPES:
        raise SdropError(EDTYPE, "sdrop_producer")
    if bias is not None and (bias.dtype != torch.float32 or tuple(bias.shape) != (K,)):
        raise ValueError("bias must be fp32 with one value per output column")
    if preact is True:
        preact = torch.zeros((M, K), dtype=out_dtype, device=H.device)
    if preact is not None and (tuple(preact.shape) != (M, K) or preact.dtype != out_dtype):
        raise ValueError("preact has the wrong shape or dtype")
    (ph, ldh), (pw, ldw), (po, ldo) = _mat(H, "H"), _mat(W0, "W0"), _mat(out, "out")
    pz = ctypes.c_void_p(0)
    if preact is not None:
        pz, ldz = _mat(preact, "preact")
        if ldz != ldo:
            raise ValueError("preact must have the output's leading dimension")
    args = (ph, pw, _dev(bias, "bias") if bias is not None else ctypes.c_void_p(0), _dev(mask.buf, "mask"), po, pz,
            M, N0, K, mask.BM, mask.BK, mask.p, int(act), _DTYPES[dtype], _DTYPES[out_dtype], _stream())
    if (ldh, ldw, ldo) == (N0, N0, K):
        rc = lib().sdrop_producer(*args)
    else:
        rc = lib().sdrop_producer_ex(*args, ldh, ldw, ldo)
    _check(rc, "sdrop_producer")
    return out if preact is None else (out, preact)


def bias_grad_workspace_bytes(M, K, BM, BK):
    return int(lib().sdrop_bias_grad_workspace_bytes(M, K, BM, BK))


def sdrop_bias_grad(dZ, mask, out=None, ws=None):
    """db[k] = sum_r (dZ . m')[r, k], fp32 [K]: the bias gradient of the layer before the dropout
    (Section 4.3, closing remark); dZ [M, K] fp16 / bf16 with contiguous rows (a leading dimension is allowed)."""
    M, K = dZ.shape
    if (M, K) != (mask.M, mask.K):
        raise SdropError(ESHAPE, "sdrop_bias_grad")
    if dZ.dtype not in (torch.float16, torch.bfloat16):
        raise SdropError(EDTYPE, "sdrop_bias_grad")
    if out is None:
        out = torch.empty(K, dtype=torch.float32, device=dZ.device)
    elif tuple(out.shape) != (K,) or out.dtype != torch.float32:
        raise ValueError("out must be fp32 with one value per column")
    need = bias_grad_workspace_bytes(M, K, mask.BM, mask.BK)
    if ws is None and need:
        ws = torch.empty(need, dtype=torch.uint8, device=dZ.device)
    ptr, ld = _mat(dZ, "dZ")
    rc = lib().sdrop_bias_grad(ptr, _dev(mask.buf, "mask"), _dev(out, "out"), M, K, mask.BM, mask.BK,
                               _DTYPES[dZ.dtype], ld,
                               ctypes.c_void_p(ws.data_ptr()) if ws is not None else ctypes.c_void_p(0),
                               ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(rc, "sdrop_bias_grad")
    return out
