"""A whole step (mask, forward, dX, dW: arxiv 2411.01238 Section 3.1-3.2) captured in a HIP graph
must give, on every replay, exactly what the same calls give eagerly: the library enqueues only
kernels (no memset nodes, no host-side state that a replay would miss)."""
import pytest
import torch

from paper_2411_01238_amd import sdrop
from paper_2411_01238_amd.workloads import make_custom

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p", [
    (1024, 1024, 512, 128, 128, "bf16", 0.5),     # persistent kernels for all three products
    (2048, 256, 264, 64, 64, "f16", 0.5),         # per-tile kernels, ragged N, dW as split parts + a summing pass
])
def test_graph_replays_equal_eager(M, K, N, BM, BK, dtype, p):
    print("graph", M, K, N, BM, BK, dtype, p, flush=True)
    X, W, dY = (t.cuda() for t in make_custom(M, K, N, dtype, seed=5))
    td = X.dtype
    Y = torch.empty((M, N), dtype=td, device="cuda")
    dX = torch.empty((M, K), dtype=td, device="cuda")
    dW = torch.empty((K, N), dtype=td, device="cuda")
    m = sdrop.Mask(M, K, BM, BK, p)
    need = sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, td, td)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def step():
        sdrop.sdrop_mask(M, K, BM, BK, p, 3, 1, out=m)
        sdrop.sdrop_fwd(X, W, m, out=Y)
        sdrop.sdrop_bwd_dx(dY, W, m, out=dX)
        sdrop.sdrop_bwd_dw(X, dY, m, out=dW, ws=ws)

    step()
    torch.cuda.synchronize()
    ref = (Y.clone(), dX.clone(), dW.clone())
    ref_bits = m.bits().clone()
    ref_lists = {k: v.clone() for k, v in m.lists().items()}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                    # warm-up on the capturing stream's side
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for _ in range(4):
        # eager work and a synchronisation between replays; outputs and the mask object wiped
        Y.fill_(7.0); dX.fill_(7.0); dW.fill_(7.0); m.buf.zero_(); ws.fill_(255)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, ref[0]) and torch.equal(dX, ref[1]) and torch.equal(dW, ref[2])
        # the mask object: its bits and every list (the lists' unused tails are not written)
        assert torch.equal(m.bits(), ref_bits)
        for k, v in m.lists().items():
            assert torch.equal(v, ref_lists[k]), k


@pytest.mark.parametrize("M,K,N,BM,BK,dtype,p", [
    (1024, 1024, 512, 128, 128, "bf16", 0.5),     # one-launch backward, persistent producer
    (1536, 256, 512, 128, 128, "f16", 0.3),       # one-launch backward whose dW part is split and summed
    (512, 768, 328, 128, 64, "bf16", 0.4),        # per-tile kernels, ragged N: the backward is two launches
])
def test_graph_of_the_sparse_block_replays_equal_eager(M, K, N, BM, BK, dtype, p):
    # mask, producing layer (with its second output), forward, both gradients in one call, gated dX
    print("graph block", M, K, N, BM, BK, dtype, p, flush=True)
    X, W, dY = (t.cuda() for t in make_custom(M, K, N, dtype, seed=6))
    td = X.dtype
    g0 = torch.Generator(device="cpu")
    g0.manual_seed(1)
    b0 = torch.randn(K, generator=g0).cuda()
    outs = {n: torch.empty(s, dtype=td, device="cuda") for n, s in
            (("Xh", (M, K)), ("Z", (M, K)), ("Y", (M, N)), ("dX", (M, K)), ("dW", (K, N)), ("dZ", (M, K)))}
    m = sdrop.Mask(M, K, BM, BK, p)
    ws = torch.empty(max(sdrop.workspace_bytes(sdrop.OP_BWD_DW, M, K, N, BM, BK, td, td), 16), dtype=torch.uint8, device="cuda")

    def step():
        sdrop.sdrop_mask(M, K, BM, BK, p, 4, 2, out=m)
        sdrop.sdrop_producer(dY, W, b0, m, act=sdrop.ACT_GELU_ERF, out=outs["Xh"], preact=outs["Z"])
        sdrop.sdrop_fwd(outs["Xh"], W, m, out=outs["Y"])
        sdrop.sdrop_bwd(dY, W, X, m, out_dx=outs["dX"], out_dw=outs["dW"], ws=ws)
        sdrop.sdrop_bwd_dx_ex(dY, W, m, relu_mask=outs["Z"], gate_mode=sdrop.GATE_GELU_ERF, out=outs["dZ"])

    def wipe():
        for o in outs.values():
            o.fill_(7.0)
        m.buf.zero_()
        ws.fill_(255)

    wipe()
    step()
    torch.cuda.synchronize()
    ref = {n: o.clone() for n, o in outs.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for _ in range(3):
        wipe()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n, o in outs.items():
            assert torch.equal(o, ref[n]), n
