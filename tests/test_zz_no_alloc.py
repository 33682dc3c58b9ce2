"""The entry point that allocates nothing (sdrop_bwd_dw_static), through the raw C ABI, against
sdrop_bwd_dw: bit-identical outputs on two calls in a row, the second on a smaller problem (the
library's own scratch memory then still holds the first call's planes), and a clear error for a
problem whose planes do not fit."""
import ctypes

import pytest
import torch

from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom

pytestmark = pytest.mark.gpu


def _case(M, K, N, BM, BK, dtype, p, seed):
    print("no-alloc case %dx%dx%d blocks %dx%d %s p=%.1f" % (M, K, N, BM, BK, dtype, p), flush=True)
    L = sdrop.lib()
    X, _, dY = make_custom(M, K, N, dtype, seed=seed)
    Xg, dYg = X.cuda(), dY.cuda()
    m = sdrop.sdrop_mask(M, K, BM, BK, p, 7, seed)
    td = Xg.dtype
    need = sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, td, td)
    assert 0 < need <= sdrop.STATIC_SCRATCH_BYTES, "the case must use a split reduction that fits"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    code = sdrop._DTYPES[td]
    vp = ctypes.c_void_p
    for out_dtype in (td, torch.float32):
        ocode = sdrop._DTYPES[out_dtype]
        ref = torch.full((K, N), float("nan"), dtype=out_dtype, device="cuda")
        got = torch.full((K, N), float("nan"), dtype=out_dtype, device="cuda")
        st = sdrop._stream()
        rc = L.sdrop_bwd_dw(vp(Xg.data_ptr()), vp(dYg.data_ptr()), vp(m.buf.data_ptr()), vp(ref.data_ptr()),
                            M, K, N, BM, BK, p, code, ocode, vp(ws.data_ptr()), need, st)
        assert rc == sdrop.OK
        rc = L.sdrop_bwd_dw_static(vp(Xg.data_ptr()), vp(dYg.data_ptr()), vp(m.buf.data_ptr()), vp(got.data_ptr()),
                                   M, K, N, BM, BK, p, code, ocode, st)
        assert rc == sdrop.OK
        torch.cuda.synchronize()
        assert torch.isfinite(ref).all().item()
        assert torch.equal(got, ref), "sdrop_bwd_dw_static differs from sdrop_bwd_dw"


def test_two_calls_in_a_row_second_smaller():
    _case(16384, 3072, 768, 128, 64, "bf16", 0.1, 1)    # 8 parts of 9 MiB planes
    _case(2048, 512, 256, 128, 128, "bf16", 0.3, 2)     # a smaller problem right after it
    _case(8192, 1024, 1024, 64, 64, "f16", 0.5, 3)


def test_too_large_is_refused_before_anything_is_enqueued():
    L = sdrop.lib()
    # 16 parts of 3072 x 768 fp32 planes: 144 MiB
    M, K, N, BM, BK = 65536, 3072, 768, 128, 128
    td = torch.bfloat16
    need = sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, td, td)
    if need <= sdrop.STATIC_SCRATCH_BYTES:
        pytest.skip("this device's CU count gives that shape a small workspace")
    X = torch.zeros((M, K), dtype=td, device="cuda")
    dY = torch.zeros((M, N), dtype=td, device="cuda")
    m = sdrop.sdrop_mask(M, K, BM, BK, 0.5, 0, 0)
    out = torch.full((K, N), 3.0, dtype=td, device="cuda")
    vp = ctypes.c_void_p
    rc = L.sdrop_bwd_dw_static(vp(X.data_ptr()), vp(dY.data_ptr()), vp(m.buf.data_ptr()), vp(out.data_ptr()),
                               M, K, N, BM, BK, 0.5, sdrop.BF16, sdrop.BF16, sdrop._stream())
    assert rc == sdrop.EWORKSPACE
    torch.cuda.synchronize()
    assert (out == 3.0).all().item()
