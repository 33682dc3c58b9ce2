"""Nothing outside a buffer is written: every output, the mask object and the workspace of each entry point sit
between guard regions that must come back untouched.  The shapes are those whose address arithmetic has edges:
N that is not a multiple of the 256-wide tile or of the 64-wide reduction slice (eq. 1-3 of arxiv 2411.01238,
Section 3.1, with a ragged last tile column or a ragged last slice), a language-model head of 72 columns, a
single block row, 64-row blocks, fp32 outputs, a split eq. 3."""
import pytest
import torch

from paper_2411_01238_amd import sdrop

pytestmark = pytest.mark.gpu

GUARD = 1 << 16       # bytes before and after each buffer
FILL = 0xA5


class Guarded:
    """A tensor of `shape`/`dtype` (or raw bytes) in the middle of a larger allocation filled with FILL."""

    def __init__(self, nbytes):
        nbytes = (nbytes + 255) // 256 * 256
        self.raw = torch.full((GUARD + nbytes + GUARD,), FILL, dtype=torch.uint8, device="cuda")
        self.body = self.raw[GUARD:GUARD + nbytes]

    def view(self, shape, dtype):
        n = 1
        for s in shape:
            n *= s
        return self.body[:n * torch.empty((), dtype=dtype).element_size()].view(dtype).view(shape)

    def intact(self):
        return bool((self.raw[:GUARD] == FILL).all().item()) and bool((self.raw[-GUARD:] == FILL).all().item())


SHAPES = [
    # M, K, N, BM, BK, dtype
    (4096, 1024, 72, 128, 128, torch.bfloat16),      # 72 columns: ragged tile column, ragged slice (72 = 64 + 8)
    (4096, 1024, 72, 64, 64, torch.float16),
    (1024, 1024, 264, 128, 128, torch.bfloat16),     # one whole tile column and 8 columns more
    (128, 4096, 1000, 128, 128, torch.float16),      # a single block row
    (4096, 128, 520, 128, 128, torch.bfloat16),      # a single block column
    (2048, 2048, 256, 128, 64, torch.bfloat16),
    (4096, 4096, 4096, 128, 128, torch.bfloat16),    # the pair list, the one-launch backward, the seeded forward
]


@pytest.mark.parametrize("M,K,N,BM,BK,dtype", SHAPES)
@pytest.mark.parametrize("out32", [False, True])
def test_no_entry_point_writes_outside_its_buffers(M, K, N, BM, BK, dtype, out32):
    print("guard case", M, K, N, BM, BK, dtype, out32, flush=True)
    p = 0.5
    od = torch.float32 if out32 else dtype
    esz = 4 if out32 else 2
    g = torch.Generator(device="cuda").manual_seed(1)
    X = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32).to(dtype)
    W = torch.randn((K, N), generator=g, device="cuda", dtype=torch.float32).to(dtype)
    dY = torch.randn((M, N), generator=g, device="cuda", dtype=torch.float32).to(dtype)
    bufs = {}

    def buf(name, nbytes):
        bufs[name] = Guarded(nbytes)
        return bufs[name]

    m = sdrop.Mask(M, K, BM, BK, p)
    m.buf = buf("mask of sdrop_mask", sdrop.mask_bytes(M, K, BM, BK)).body[:sdrop.mask_bytes(M, K, BM, BK)]
    sdrop.sdrop_mask(M, K, BM, BK, p, 3, 1, out=m)
    m2 = sdrop.Mask(M, K, BM, BK, p)
    m2.buf = buf("mask of sdrop_fwd_seeded", sdrop.mask_bytes(M, K, BM, BK)).body[:sdrop.mask_bytes(M, K, BM, BK)]
    Y2 = buf("Y of sdrop_fwd_seeded", M * N * esz).view((M, N), od)
    sdrop.sdrop_fwd_seeded(X, W, BM, BK, p, 3, 1, mask=m2, out_dtype=od, out=Y2)
    Y = buf("Y", M * N * esz).view((M, N), od)
    sdrop.sdrop_fwd(X, W, m, out_dtype=od, out=Y)
    dX = buf("dX", M * K * esz).view((M, K), od)
    sdrop.sdrop_bwd_dx(dY, W, m, out_dtype=od, out=dX)
    need = sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, dtype, od)
    ws = buf("workspace of sdrop_bwd_dw", max(need, 256)).body
    dW = buf("dW", K * N * esz).view((K, N), od)
    sdrop.sdrop_bwd_dw(X, dY, m, out_dtype=od, out=dW, ws=ws if need else None)
    dX2 = buf("dX of sdrop_bwd", M * K * esz).view((M, K), od)
    dW2 = buf("dW of sdrop_bwd", K * N * esz).view((K, N), od)
    ws2 = buf("workspace of sdrop_bwd", max(need, 256)).body
    sdrop.sdrop_bwd(dY, W, X, m2, out_dtype=od, out_dx=dX2, out_dw=dW2, ws=ws2 if need else None)
    # the same products with the weight as [N,K] (in place where the kernels have a form for it, else through the
    # workspace), outputs and workspace guarded as well
    Wt = W.t().contiguous()
    import ctypes
    code, ocode = sdrop._DTYPES[dtype], sdrop._DTYPES[od]
    epi = sdrop._epilogue(sdrop.SCALE_DROPOUT, sdrop.ACT_NONE, None, None, N, (M, N), dtype, w_layout=sdrop.W_NK)
    need_nk = max(sdrop.lib().sdrop_workspace_bytes_ex(op, M, K, N, BM, BK, code, ocode, ctypes.byref(epi))
                  for op in (sdrop.OP_FWD, sdrop.OP_BWD_DX, sdrop.OP_BWD_DW))
    ws3 = buf("workspace of the [N,K] calls", max(need_nk, 256)).body
    Y3 = buf("Y, W as [N,K]", M * N * esz).view((M, N), od)
    sdrop.sdrop_fwd_ex(X, Wt, m, out_dtype=od, out=Y3, ws=ws3, w_layout=sdrop.W_NK)
    dX3 = buf("dX, W as [N,K]", M * K * esz).view((M, K), od)
    sdrop.sdrop_bwd_dx_ex(dY, Wt, m, out_dtype=od, out=dX3, ws=ws3, w_layout=sdrop.W_NK)
    dW3 = buf("dW as [N,K]", K * N * esz).view((N, K), od)
    sdrop.sdrop_bwd_dw_ex(X, dY, m, out_dtype=od, out=dW3, ws=ws3, w_layout=sdrop.W_NK)
    torch.cuda.synchronize()
    assert torch.equal(Y3, Y) and torch.equal(dX3, dX) and torch.equal(dW3, dW.t())
    assert sdrop.status() == 0
    for name, b in bufs.items():
        assert b.intact(), "%s: bytes outside the buffer were written" % name
    assert torch.equal(Y, Y2) and torch.equal(dX, dX2) and torch.equal(dW, dW2)
