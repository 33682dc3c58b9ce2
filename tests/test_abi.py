"""CPU-only checks of the C-ABI library: it loads, exports what the header declares,
and its host-side argument checks answer before anything is enqueued."""
import ctypes
import os
import re

import pytest

from paper_2411_01238_amd import sdrop

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sdrop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdrop_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sdrop.lib()
    names = _declared()
    assert set(names) == set(sdrop.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_strerror_and_codes():
    assert sdrop.strerror(sdrop.OK) == "ok"
    for c in range(1, 7):
        assert len(sdrop.strerror(c)) > 3
    assert "unknown" in sdrop.strerror(99)


def test_tuning_knobs_reject_bad_arguments():
    L = sdrop.lib()
    assert L.sdrop_set_tuning(99, 1) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, -1) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_PERSISTENT_GROUPS_PER_CU, sdrop.DX_PERSISTENT_GROUPS_PER_CU_DEFAULT) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_TILE_WIDTH, 64) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_TILE_WIDTH, 256) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_TILE_WIDTH, 0) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_BWD_FUSED, 2) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_BWD_FUSED, -1) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_BWD_FUSED, 0) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_BWD_FUSED, 1) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_PAIRS, 3) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_PAIRS, 2) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_DX_PAIRS, 0) == sdrop.OK
    assert L.sdrop_set_tuning(sdrop.TUNE_DW64_PERSISTENT_SLICES, -1) == sdrop.EINVAL
    assert L.sdrop_set_tuning(sdrop.TUNE_DW64_PERSISTENT_SLICES, 16) == sdrop.OK


def test_mask_layout_regions_do_not_overlap():
    for (M, K, BM, BK) in ((256, 256, 64, 64), (4096, 4096, 128, 128), (65536, 4096, 128, 128),
                           (16384, 3072, 128, 64), (64, 64 * 130, 64, 64)):
        L = sdrop.mask_layout(M, K, BM, BK)
        MB, KB = M // BM, K // BK
        assert (L.MB, L.KB, L.words_per_row) == (MB, KB, (KB + 63) // 64)
        regions = [(0, 256), (L.off_bits, 8 * MB * L.words_per_row), (L.off_row_ptr, 4 * (MB + 1)),
                   (L.off_col_idx, 4 * MB * KB), (L.off_blk_row, 4 * MB * KB), (L.off_col_ptr, 4 * (KB + 1)),
                   (L.off_row_idx, 4 * MB * KB), (L.off_row_order, 4 * MB), (L.off_col_order, 4 * KB),
                   (L.off_loc_row, 4 * MB * KB), (L.off_loc_col, 4 * MB * KB), (L.off_units, 4 * MB * KB)]
        end = 0
        for off, size in regions:
            assert off >= end and off % 16 == 0
            end = off + size
        assert L.total_bytes >= end
        assert sdrop.mask_bytes(M, K, BM, BK) == L.total_bytes


def test_bad_shapes_have_no_layout():
    assert sdrop.mask_bytes(100, 256, 64, 64) == 0        # BM does not divide M
    assert sdrop.mask_bytes(256, 256, 48, 64) == 0        # unsupported block
    assert sdrop.mask_bytes(0, 256, 64, 64) == 0
    with pytest.raises(sdrop.SdropError) as e:
        sdrop.mask_layout(256, 200, 64, 64)
    assert e.value.code == sdrop.ESHAPE


def test_host_side_argument_errors_return_before_any_launch():
    L = sdrop.lib()
    buf = ctypes.create_string_buffer(1 << 16)   # host memory: never dereferenced by these calls
    addr = (ctypes.addressof(buf) + 15) // 16 * 16
    p = ctypes.c_void_p(addr)
    null = ctypes.c_void_p(0)
    assert L.sdrop_mask(null, 1 << 16, 256, 256, 64, 64, 0.5, 0, 0, null) == sdrop.EINVAL
    assert L.sdrop_mask(p, 1 << 16, 256, 256, 64, 64, 1.5, 0, 0, null) == sdrop.EINVAL
    assert L.sdrop_mask(p, 1 << 16, 256, 256, 64, 64, float("nan"), 0, 0, null) == sdrop.EINVAL
    assert L.sdrop_mask(p, 1 << 16, 250, 256, 64, 64, 0.5, 0, 0, null) == sdrop.ESHAPE
    assert L.sdrop_mask(p, 16, 256, 256, 64, 64, 0.5, 0, 0, null) == sdrop.EWORKSPACE
    assert L.sdrop_mask(ctypes.c_void_p(addr + 4), 1 << 16, 256, 256, 64, 64, 0.5, 0, 0, null) == sdrop.EALIGN
    assert L.sdrop_mask_from_bits(p, 1 << 16, 256, 256, 64, 64, null, null) == sdrop.EINVAL
    assert L.sdrop_mask_split(p, 1 << 16, 256, 256, 64, 64, 0, 1, 0.5, 0, 0, null) == sdrop.EINVAL
    assert L.sdrop_mask_split(p, 1 << 16, 256, 256, 64, 64, 3, 1, 0.5, 0, 0, null) == sdrop.ESHAPE   # 4 block rows
    assert L.sdrop_mask_split(p, 1 << 16, 256, 256, 64, 64, 2, 8, 0.5, 0, 0, null) == sdrop.ESHAPE
    for name in ("sdrop_fwd", "sdrop_bwd_dx", "sdrop_bwd_dw"):
        f = getattr(L, name)
        ok = (p, p, p, p, 256, 256, 256, 64, 64, 0.5, sdrop.F16, sdrop.F16, null, 0, null)

        def call(**kw):
            a = list(ok)
            for k, v in kw.items():
                a[int(k[1:])] = v
            return f(*a)
        assert call(a0=null) == sdrop.EINVAL
        assert call(a3=null) == sdrop.EINVAL
        assert call(a9=-0.1) == sdrop.EINVAL
        assert call(a4=255) == sdrop.ESHAPE
        assert call(a6=250) == sdrop.ESHAPE           # N not a multiple of 8
        assert call(a7=32) == sdrop.ESHAPE
        assert call(a10=sdrop.F32) == sdrop.EDTYPE
        assert call(a11=sdrop.BF16) == sdrop.EDTYPE   # out_dtype must be the input type or fp32
        assert call(a1=ctypes.c_void_p(addr + 8)) == sdrop.EALIGN


def test_mask_bits_rejects_null_arguments_on_the_host():
    import ctypes
    L = sdrop.lib()
    buf = (ctypes.c_uint64 * 4)()
    assert L.sdrop_mask_bits(None, buf, 4, None, None) == sdrop.EINVAL
    # neither output asked for (the mask pointer is never dereferenced on the host)
    assert L.sdrop_mask_bits(ctypes.c_void_p(4096), None, 0, None, None) == sdrop.EINVAL


def test_fused_backward_checks_both_products_before_any_launch():
    L = sdrop.lib()
    buf = ctypes.create_string_buffer(1 << 16)
    addr = (ctypes.addressof(buf) + 15) // 16 * 16
    p = ctypes.c_void_p(addr)
    null = ctypes.c_void_p(0)
    ok = (p, p, p, p, p, p, 2048, 256, 264, 64, 64, 0.5, sdrop.F16, sdrop.F16, null, 0, null)

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return L.sdrop_bwd(*a)
    for i in range(6):
        assert call(**{"a%d" % i: null}) == sdrop.EINVAL
        assert call(**{"a%d" % i: ctypes.c_void_p(addr + 8)}) == sdrop.EALIGN
    assert call(a11=1.5) == sdrop.EINVAL
    assert call(a6=2047) == sdrop.ESHAPE
    assert call(a8=250) == sdrop.ESHAPE
    assert call(a12=sdrop.F32) == sdrop.EDTYPE
    # few output tiles and long columns: the weight gradient is split, so a workspace is required
    assert L.sdrop_workspace_bytes(sdrop.OP_BWD_DW, 2048, 256, 264, 64, 64, sdrop.F16, sdrop.F16) > 0
    assert call() == sdrop.EWORKSPACE


def test_tail_arguments_are_checked_on_the_host():
    L = sdrop.lib()
    buf = ctypes.create_string_buffer(1 << 16)
    addr = (ctypes.addressof(buf) + 15) // 16 * 16
    p = ctypes.c_void_p(addr)
    null = ctypes.c_void_p(0)
    # 64 x 64 blocks over 256 x 16384: 256 output tiles for dW, so no workspace is asked for
    base = (p, p, p, p, 256, 16384, 256, 64, 64, 0.5, sdrop.F16, sdrop.F16, null, 0, null)

    def epi(scale_mode=sdrop.SCALE_DROPOUT, act=sdrop.ACT_NONE, bias=None, relu_mask=None):
        e = sdrop.Epilogue()
        e.scale_mode, e.act, e.bias, e.relu_mask = scale_mode, act, bias, relu_mask
        return ctypes.byref(e)
    for name in ("sdrop_fwd_ex", "sdrop_bwd_dx_ex", "sdrop_bwd_dw_ex"):
        f = getattr(L, name)
        assert f(*base[:3], null, *base[4:], epi()) == sdrop.EINVAL          # the plain checks still apply
        assert f(*base, epi(scale_mode=2)) == sdrop.EINVAL
        assert f(*base, epi(act=4)) == sdrop.EINVAL
        assert f(*base, epi(act=-1)) == sdrop.EINVAL
        e = sdrop.Epilogue()
        e.gate_mode = 3
        assert f(*base, ctypes.byref(e)) == sdrop.EINVAL
    for name in ("sdrop_fwd_ex", "sdrop_bwd_dx_ex"):
        f = getattr(L, name)
        assert f(*base, epi(bias=addr + 4)) == sdrop.EALIGN
        assert f(*base, epi(relu_mask=addr + 8)) == sdrop.EALIGN
    # leading dimensions: at least the row length, a multiple of 8
    def epi_ld(a=0, b=0, o=0):
        e = sdrop.Epilogue()
        e.scale_mode, e.act, e.bias, e.relu_mask, e.ld_a, e.ld_b, e.ld_out = 0, 0, None, None, a, b, o
        return ctypes.byref(e)
    for name in ("sdrop_fwd_ex", "sdrop_bwd_dx_ex", "sdrop_bwd_dw_ex"):
        f = getattr(L, name)
        for kw in (dict(a=8), dict(b=248), dict(o=16), dict(a=16384 + 4), dict(b=1 << 25)):
            assert f(*base, epi_ld(**kw)) == sdrop.ESHAPE, (name, kw)
    # the gradient of the weights takes a scale and leading dimensions only
    f = L.sdrop_bwd_dw_ex
    assert f(*base, epi(act=sdrop.ACT_RELU)) == sdrop.EINVAL
    assert f(*base, epi(bias=addr)) == sdrop.EINVAL
    assert f(*base, epi(relu_mask=addr)) == sdrop.EINVAL
    # the producer: same checks as eq. (2), plus the activation
    g = L.sdrop_producer
    ok = (p, p, null, p, p, null, 256, 256, 256, 64, 64, 0.5, sdrop.ACT_RELU, sdrop.F16, sdrop.F16, null)
    assert g(*ok[:12], 7, *ok[13:]) == sdrop.EINVAL
    assert g(null, *ok[1:]) == sdrop.EINVAL
    assert g(*ok[:6], 250, *ok[7:]) == sdrop.ESHAPE
    assert g(*ok[:2], ctypes.c_void_p(addr + 4), *ok[3:]) == sdrop.EALIGN
    assert g(*ok[:5], ctypes.c_void_p(addr + 8), *ok[6:]) == sdrop.EALIGN      # the second output


def test_workspace_size_is_a_whole_number_of_fp32_planes():
    # only dW asks for a workspace: `parts` fp32 planes of K x N, parts a power of two up to 16, none
    # when K/BK * ceil(N/256) output tiles already fill the chip (256 CUs assumed without a device)
    L = sdrop.lib()
    for (M, K, N, BM, BK) in ((4096, 4096, 4096, 128, 128), (65536, 4096, 1024, 128, 128), (8192, 1024, 1024, 64, 64),
                              (16384, 3072, 768, 128, 64), (2048, 256, 264, 64, 64), (256, 256, 8, 128, 128)):
        for op in (sdrop.OP_FWD, sdrop.OP_BWD_DX):
            assert L.sdrop_workspace_bytes(op, M, K, N, BM, BK, sdrop.BF16, sdrop.BF16) == 0
        b = L.sdrop_workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, sdrop.BF16, sdrop.BF16)
        assert b % (K * N * 4) == 0
        parts = b // (K * N * 4)
        tiles = (K // BK) * ((N + 255) // 256)
        assert parts in (0, 2, 4, 8, 16)
        if tiles >= 304:
            assert parts == 0
        assert parts <= max((M // BM) // 4, 1) or parts == 0
    assert L.sdrop_workspace_bytes(sdrop.OP_BWD_DW, 100, 256, 256, 64, 64, sdrop.BF16, sdrop.BF16) == 0   # bad shape


def test_bias_gradient_arguments_are_checked_on_the_host():
    L = sdrop.lib()
    buf = ctypes.create_string_buffer(1 << 16)   # host memory: never dereferenced by these calls
    addr = (ctypes.addressof(buf) + 15) // 16 * 16
    p, null = ctypes.c_void_p(addr), ctypes.c_void_p(0)
    ok = (p, p, p, 65536, 1024, 128, 128, sdrop.BF16, 0, null, 0, null)

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return L.sdrop_bias_grad(*a)
    assert call(a0=null) == sdrop.EINVAL and call(a1=null) == sdrop.EINVAL and call(a2=null) == sdrop.EINVAL
    assert call(a3=65500) == sdrop.ESHAPE and call(a5=32) == sdrop.ESHAPE
    assert call(a7=sdrop.F32) == sdrop.EDTYPE
    assert call(a2=ctypes.c_void_p(addr + 4)) == sdrop.EALIGN
    assert call(a8=1000) == sdrop.ESHAPE and call(a8=1028) == sdrop.ESHAPE     # shorter than a row; not a multiple of 8
    # 512 block rows, 8 block columns: the lists are cut into parts, whose fp32 rows need a workspace
    need = L.sdrop_bias_grad_workspace_bytes(65536, 1024, 128, 128)
    assert need > 0 and need % (1024 * 4) == 0 and need // (1024 * 4) <= 64
    assert call() == sdrop.EWORKSPACE
    assert call(a9=ctypes.c_void_p(addr + 4), a10=need) == sdrop.EWORKSPACE
    # at most one part per block row; none for a bad shape
    assert L.sdrop_bias_grad_workspace_bytes(128, 1024, 128, 128) == 0
    assert L.sdrop_bias_grad_workspace_bytes(100, 1024, 128, 128) == 0


def test_new_entry_points_check_their_arguments_on_the_host():
    L = sdrop.lib()
    buf = ctypes.create_string_buffer(1 << 16)
    addr = (ctypes.addressof(buf) + 15) // 16 * 16
    p = ctypes.c_void_p(addr)
    null = ctypes.c_void_p(0)
    # sdrop_bwd_ex: leading dimensions of dY, W, X, dX, dW
    ok = (p, p, p, p, p, p, 2048, 256, 264, 64, 64, 0.5, sdrop.F16, sdrop.F16, null, 0, null)
    assert L.sdrop_bwd_ex(*ok, 0, 0, 0, 0, 0, sdrop.W_KN) == sdrop.EWORKSPACE          # as sdrop_bwd: the split needs a workspace
    assert L.sdrop_bwd_ex(*ok, 256, 0, 0, 0, 0, sdrop.W_KN) == sdrop.ESHAPE            # dY has 264 columns
    assert L.sdrop_bwd_ex(*ok, 0, 0, 260, 0, 0, sdrop.W_KN) == sdrop.ESHAPE            # not a multiple of 8
    assert L.sdrop_bwd_ex(*ok, 0, 0, 0, 0, (1 << 24) + 8, sdrop.W_KN) == sdrop.ESHAPE
    assert L.sdrop_bwd_ex(*ok, 0, 0, 0, 0, 0, 5) == sdrop.EINVAL                       # no such layout
    assert L.sdrop_bwd_ex(*ok, 0, 0, 0, 0, 0, sdrop.W_NK) == sdrop.EWORKSPACE
    assert L.sdrop_bwd_ex(*ok, 0, 0, 0, 0, 128, sdrop.W_NK) == sdrop.ESHAPE            # dW[N,K] has 256 columns
    # sdrop_producer_ex
    okp = (p, p, null, p, p, null, 256, 256, 256, 64, 64, 0.5, sdrop.ACT_RELU, sdrop.F16, sdrop.F16, null)
    assert L.sdrop_producer_ex(*okp, 128, 0, 0) == sdrop.ESHAPE
    assert L.sdrop_producer_ex(*okp, 0, 0, 260) == sdrop.ESHAPE
    # the weight's layout: bad enum, the larger workspace
    e = sdrop.Epilogue()
    e.scale_mode, e.act, e.gate_mode, e.w_layout = 0, 0, 0, 7
    okf = (p, p, p, p, 256, 256, 256, 64, 64, 0.5, sdrop.F16, sdrop.F16, null, 0, null)
    assert L.sdrop_fwd_ex(*okf, ctypes.byref(e)) == sdrop.EINVAL
    e.w_layout, e.kept_fraction = sdrop.W_KN, 1.5
    assert L.sdrop_fwd_ex(*okf, ctypes.byref(e)) == sdrop.EINVAL
    e.w_layout, e.kept_fraction = sdrop.W_NK, 0.25
    assert L.sdrop_fwd_ex(*okf, ctypes.byref(e)) == sdrop.EWORKSPACE
    assert L.sdrop_workspace_bytes_ex(sdrop.OP_FWD, 256, 256, 512, 64, 64, sdrop.F16, sdrop.F16, ctypes.byref(e)) == 256 * 512 * 2
    assert L.sdrop_workspace_bytes_ex(sdrop.OP_BWD_DX, 256, 256, 512, 64, 64, sdrop.F16, sdrop.F32, ctypes.byref(e)) == 256 * 512 * 2
    planes = L.sdrop_workspace_bytes(sdrop.OP_BWD_DW, 2048, 256, 264, 64, 64, sdrop.F16, sdrop.F32)
    assert L.sdrop_workspace_bytes_ex(sdrop.OP_BWD_DW, 2048, 256, 264, 64, 64, sdrop.F16, sdrop.F32, ctypes.byref(e)) == planes + 256 * 264 * 4
    assert L.sdrop_workspace_bytes_ex(sdrop.OP_BWD_DW, 2048, 256, 264, 64, 64, sdrop.F16, sdrop.F32, None) == planes
    # sdrop_fwd_seeded
    oks = (p, p, p, 1 << 16, p, 256, 256, 256, 64, 64, 0.5, 1, 2, sdrop.F16, sdrop.F16, null)
    assert L.sdrop_fwd_seeded(*(oks[:2] + (null,) + oks[3:])) == sdrop.EINVAL
    assert L.sdrop_fwd_seeded(*(oks[:3] + (64,) + oks[4:])) == sdrop.EWORKSPACE
    assert L.sdrop_fwd_seeded(*(oks[:10] + (1.5,) + oks[11:])) == sdrop.EINVAL
    assert L.sdrop_fwd_seeded(*(oks[:7] + (250,) + oks[8:])) == sdrop.ESHAPE
    # sdrop_fwd_seeded_ex: the layout and the leading dimensions only
    okx = oks[:15] + (null, 0, null)
    e2 = sdrop.Epilogue()
    e2.scale_mode, e2.act, e2.gate_mode, e2.w_layout = 0, 0, 0, sdrop.W_NK
    assert L.sdrop_fwd_seeded_ex(*okx, ctypes.byref(e2)) == sdrop.EWORKSPACE               # room for the transposed copy
    e2.w_layout, e2.act = sdrop.W_KN, sdrop.ACT_RELU
    assert L.sdrop_fwd_seeded_ex(*okx, ctypes.byref(e2)) == sdrop.EINVAL                   # no tail in this call
    e2.act, e2.ld_a = sdrop.ACT_NONE, 128
    assert L.sdrop_fwd_seeded_ex(*okx, ctypes.byref(e2)) == sdrop.ESHAPE                   # X has 256 columns
    assert L.sdrop_fwd_seeded_ex(*(okx[:2] + (null,) + okx[3:]), None) == sdrop.EINVAL
    assert L.sdrop_status(None, 0, None) == sdrop.EINVAL
    # sdrop_bwd_dw_static: argument errors as sdrop_bwd_dw
    okd = (p, p, p, p, 256, 256, 256, 64, 64, 0.5, sdrop.F16, sdrop.F16, null)
    assert L.sdrop_bwd_dw_static(*((null,) + okd[1:])) == sdrop.EINVAL
    assert L.sdrop_bwd_dw_static(*(okd[:6] + (250,) + okd[7:])) == sdrop.ESHAPE
