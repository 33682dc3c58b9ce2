"""eq. (1) and eq. (3) of arxiv 2411.01238 (Section 3.1) when N is not a multiple of the 256-wide
tile and the problem has at least a chip's worth of whole tiles.  Without a tail the persistent
kernels take the ragged tile column themselves (their loaders fetch only the chunks that exist,
their epilogue stops at N); with a tail the library issues the whole tile columns and the ragged
rest as two launches.  Parity against the float64 oracle as for every other shape, the tail's
operands (bias, gate) included, which move with the columns."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom
from _util import f64, assert_close
from test_gpu_gemm import _full_parity

pytestmark = pytest.mark.gpu

CUS = 256       # MI355X


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p,seed", [
    (2048, 512, 4104, 128, 128, "bf16", 0.5, 51),   # fwd: 16 block rows x 16 whole tiles, 8 ragged columns
    (4096, 256, 2120, 64, 64, "f16", 0.3, 52),      # fwd: 64 block rows x 8 whole tiles, 72 ragged columns
    (512, 4096, 2056, 128, 128, "bf16", 0.4, 53),   # dW: 32 block columns x 8 whole tiles (fwd: too few rows, one launch)
    (4096, 1024, 1032, 64, 64, "f16", 0.5, 54),     # dW cut into parts along M as well
])
def test_products_with_whole_and_ragged_tile_columns(M, K, N, BM, BK, dtype, p, seed):
    print("ragged split", M, K, N, BM, BK, dtype, p, seed, flush=True)
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    parts = max(sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, td, td) // (K * N * 4), 1)
    whole = N // 256
    # large enough for many tiles per workgroup in at least one of the two products
    assert (M // BM) * whole >= CUS or (K // BK) * parts * whole >= CUS
    X, W, dY = make_custom(M, K, N, dtype, seed=seed)
    _full_parity(X, W, dY, BM, BK, p, seed, 0, "ragged-split(%d,%d,%d,%dx%d,%s)" % (M, K, N, BM, BK, dtype))


@pytest.mark.parametrize("out_dtype", [None, torch.float32])
def test_forward_tail_operands_move_with_the_columns(out_dtype):
    M, K, N, BM, BK, p, seed = 2048, 512, 4168, 128, 128, 0.5, 55
    print("ragged split tail", out_dtype, flush=True)
    X, W, _ = make_custom(M, K, N, "f16", seed=seed)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    bias = torch.randn(N, generator=g, dtype=torch.float32)
    gate = torch.randn(M, N, generator=g).to(torch.float16)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, 0)
    keep = orc.mask(M // BM, K // BK, p, seed, 0)
    # bias and ReLU; bias and a ReLU gate (read per 16-byte row piece for 16-bit outputs, per register quad for fp32)
    y = sdrop.sdrop_fwd_ex(X.cuda(), W.cuda(), m, act=sdrop.ACT_RELU, bias=bias.cuda(), out_dtype=out_dtype)
    ref = sb.fwd_tail(f64(X), f64(W), keep, BM, BK, p, bias=bias.numpy(), kind=sb.ACT_RELU)
    assert_close(f64(y), ref, "fwd bias + ReLU over a column split")
    y = sdrop.sdrop_fwd_ex(X.cuda(), W.cuda(), m, bias=bias.cuda(), relu_mask=gate.cuda(), out_dtype=out_dtype)
    ref = sb.fwd_tail(f64(X), f64(W), keep, BM, BK, p, bias=bias.numpy(), relu_mask=f64(gate))
    assert_close(f64(y), ref, "fwd bias + gate over a column split")
