"""sdrop_bias_grad (the bias gradient of the layer before the dropout: arxiv 2411.01238, Section 4.3,
closing remark) against the float64 oracle: column sums of dZ over the kept blocks."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from oracle import sparse_block_oracle as sb
from paper_2411_01238_amd import sdrop
from _util import f64, assert_close

pytestmark = pytest.mark.gpu


def _dz(M, K, dtype, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(M, K, generator=g).to(torch.float16 if dtype == "f16" else torch.bfloat16)


def _poison_dropped(dZ, keep, BM, BK):
    """NaN in every dropped block: they must not be read."""
    m = torch.from_numpy(np.asarray(keep)).bool().repeat_interleave(BM, 0).repeat_interleave(BK, 1)
    out = dZ.clone()
    out[~m] = float("nan")
    return out


@pytest.mark.parametrize("M,K,BM,BK,dtype,p", [
    (1024, 768, 128, 128, "bf16", 0.5),
    (640, 448, 64, 64, "f16", 0.3),
    (512, 384, 128, 64, "bf16", 0.7),
    (384, 512, 64, 128, "f16", 0.5),
    (128, 128, 128, 128, "bf16", 0.0),            # one block
    (2048, 256, 64, 128, "f16", 0.0),             # nothing dropped, long lists
    (512, 512, 128, 128, "bf16", 1.0),            # everything dropped: zeros
    (4096, 4096, 128, 128, "bf16", 0.5),          # the benchmark's size: one part per block row
    (65536, 1024, 128, 128, "bf16", 0.5),         # long lists cut into 64 parts
])
def test_matches_oracle(M, K, BM, BK, dtype, p):
    print("bias_grad", M, K, BM, BK, dtype, p, flush=True)
    keep = orc.mask(M // BM, K // BK, p, 11, 3)
    dZ = _poison_dropped(_dz(M, K, dtype, 5), keep, BM, BK)
    m = sdrop.sdrop_mask(M, K, BM, BK, p, 11, 3)
    db = sdrop.sdrop_bias_grad(dZ.cuda(), m)
    torch.cuda.synchronize()
    want = sb.bias_grad(f64(dZ), keep, BM, BK)
    if p == 1.0:
        assert torch.count_nonzero(db).item() == 0
    else:
        assert_close(f64(db), want, "db")
    # a second call gives the same bits (fixed summation order), also into a dirty output and workspace
    need = sdrop.bias_grad_workspace_bytes(M, K, BM, BK)
    ws = torch.full((max(need, 16),), 255, dtype=torch.uint8, device="cuda")
    db2 = torch.full((K,), 7.0, dtype=torch.float32, device="cuda")
    sdrop.sdrop_bias_grad(dZ.cuda(), m, out=db2, ws=ws)
    assert torch.equal(db, db2)


def test_column_range_of_a_wider_matrix():
    M, K, BM, BK, p = 768, 512, 128, 128, 0.4
    keep = orc.mask(M // BM, K // BK, p, 2, 0)
    wide = torch.randn(M, K + 256, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16).cuda()
    view = wide[:, 128:128 + K]
    m = sdrop.sdrop_mask(M, K, BM, BK, p, 2, 0)
    db = sdrop.sdrop_bias_grad(view, m)
    assert_close(f64(db), sb.bias_grad(f64(view), keep, BM, BK), "db of a column range")
    assert torch.equal(db, sdrop.sdrop_bias_grad(view.contiguous(), m))


def test_counts_rows_exactly():
    # dZ = 1: db[k] = BM * (kept blocks in k's block column), exact in fp32
    M, K, BM, BK, p = 1024, 1024, 64, 64, 0.5
    keep = np.asarray(orc.mask(M // BM, K // BK, p, 4, 1))
    m = sdrop.sdrop_mask(M, K, BM, BK, p, 4, 1)
    db = sdrop.sdrop_bias_grad(torch.ones(M, K, dtype=torch.float16, device="cuda"), m)
    np.testing.assert_array_equal(db.cpu().numpy(), np.repeat(keep.sum(axis=0) * BM, BK).astype(np.float32))


def test_foreign_mask_and_bad_arguments():
    M, K = 512, 512
    dZ = torch.ones(M, K, dtype=torch.bfloat16, device="cuda")
    other = sdrop.sdrop_mask(M, K, 64, 64, 0.5, 1, 0)
    other.BM = other.BK = 128                    # claims 128-blocks; the header says 64
    if other.buf.numel() >= sdrop.mask_bytes(M, K, 128, 128):
        db = torch.full((K,), 3.0, dtype=torch.float32, device="cuda")
        sdrop.sdrop_bias_grad(dZ, other, out=db)
        torch.cuda.synchronize()
        assert torch.all(db == 3.0)              # a mask built for another problem: nothing is written
    m = sdrop.sdrop_mask(M, K, 128, 128, 0.5, 1, 0)
    with pytest.raises(sdrop.SdropError) as e:
        sdrop.sdrop_bias_grad(dZ.float(), m)
    assert e.value.code == sdrop.EDTYPE
    with pytest.raises(sdrop.SdropError) as e:
        sdrop.sdrop_bias_grad(dZ[:256], m)
    assert e.value.code == sdrop.ESHAPE
    need = sdrop.bias_grad_workspace_bytes(M, K, 128, 128)
    if need:
        with pytest.raises(sdrop.SdropError) as e:
            sdrop.sdrop_bias_grad(dZ, m, ws=torch.empty(need - 16, dtype=torch.uint8, device="cuda"))
        assert e.value.code == sdrop.EWORKSPACE
