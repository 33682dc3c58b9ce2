"""torch.autograd wrapper over the binding: SparseDrop in front of a linear layer as one op.

Section 3.1 of arxiv 2411.01238: forward eq. (1), backward eq. (2) and (3), the block mask of
Section 3.2 drawn once per call and shared by the three products.  Everything runs in libsdrop's
kernels; this file only wires them into autograd (no arithmetic of its own besides the bias add
and the seed bookkeeping).
"""
import torch

from . import sdrop


class _SparseDropMatmul(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, w, p, BM, BK, seed, rng_stream, w_layout):
        # the mask and eq. (1) in one call (one launch for block grids up to 128 x 64); m serves the backward
        y, m = sdrop.sdrop_fwd_seeded(x, w, BM, BK, p, seed, rng_stream, w_layout=w_layout)
        ctx.save_for_backward(x, w)
        ctx.mask = m
        ctx.w_layout = w_layout
        return y

    @staticmethod
    def backward(ctx, dy):
        x, w = ctx.saved_tensors
        dy = dy.contiguous()
        wl = ctx.w_layout
        if ctx.needs_input_grad[0] and ctx.needs_input_grad[1]:
            dx, dw = sdrop.sdrop_bwd(dy, w, x, ctx.mask, w_layout=wl)      # both gradients, one launch where the shapes allow it
        else:
            dx = sdrop.sdrop_bwd_dx_ex(dy, w, ctx.mask, w_layout=wl) if ctx.needs_input_grad[0] else None
            dw = sdrop.sdrop_bwd_dw_ex(x, dy, ctx.mask, w_layout=wl) if ctx.needs_input_grad[1] else None
        return dx, dw, None, None, None, None, None, None


def sparsedrop_matmul(x, w, p, BM=128, BK=128, seed=0, rng_stream=0, weight_layout="kn"):
    """y = (x . m') w / (1 - p) with a fresh block mask m' (Bernoulli(1-p) per BM x BK block of x).

    x [M, K] and w [K, N] are fp16 / bf16 GPU tensors with contiguous rows; M % BM == 0, K % BK == 0, N % 8 == 0.
    weight_layout="nk": w is [N, K], one row per output feature (the layout of torch.nn.Linear's weight), and so is
    its gradient.
    """
    wl = {"kn": sdrop.W_KN, "nk": sdrop.W_NK}[weight_layout]
    return _SparseDropMatmul.apply(x, w, float(p), int(BM), int(BK), int(seed), int(rng_stream), wl)


_ACTS = {"relu": (sdrop.ACT_RELU, sdrop.GATE_RELU), "gelu_tanh": (sdrop.ACT_GELU_TANH, sdrop.GATE_GELU_TANH),
         "gelu": (sdrop.ACT_GELU_ERF, sdrop.GATE_GELU_ERF)}


class _SparseActBlock(torch.autograd.Function):
    """Linear -> activation -> SparseDrop -> Linear with every GEMM sparse (Section 4.3, closing remark).

    forward   X = m' . act(H W0^T + b0)          sdrop_producer (dropped blocks never computed;
                                                 for a GELU it also keeps Z = H W0^T + b0 on the kept blocks)
              Y = s X W                          eq. (1)
    backward  dZ  = s (dY W^T) . m' . act'(Z)    eq. (2) with the gate in its tail ([X > 0] for ReLU)
              dW  = s X^T dY                     eq. (3)
              dH  = dZ W0, dW0 = dZ^T H          eq. (1) / eq. (3) at scale 1 on the block-sparse dZ
              db0 = column sums of dZ            sdrop_bias_grad (kept blocks only)
    """

    @staticmethod
    def forward(ctx, h, w0, b0, w, p, BM, BK, seed, rng_stream, act):
        M, K = h.shape[0], w0.shape[0]
        act_id, gate_id = _ACTS[act]
        m = sdrop.sdrop_mask(M, K, BM, BK, p, seed, rng_stream)
        if act == "relu":
            x = sdrop.sdrop_producer(h, w0, b0, m, act=act_id)
            gate = x                    # [X > 0] is [Z > 0] on the kept blocks
        else:
            x, gate = sdrop.sdrop_producer(h, w0, b0, m, act=act_id, preact=True)
        y = sdrop.sdrop_fwd(x, w, m)
        ctx.save_for_backward(h, w0, w, x, gate)
        ctx.mask = m
        ctx.has_bias = b0 is not None
        ctx.gate_id = gate_id
        return y

    @staticmethod
    def backward(ctx, dy):
        h, w0, w, x, gate = ctx.saved_tensors
        m = ctx.mask
        dy = dy.contiguous()
        need_h, need_w0, need_b0, need_w = ctx.needs_input_grad[:4]
        dz = dh = dw0 = db0 = dw = None
        if need_h or need_w0 or (need_b0 and ctx.has_bias):
            dz = sdrop.sdrop_bwd_dx_ex(dy, w, m, relu_mask=gate, gate_mode=ctx.gate_id)
        if need_h:
            dh = sdrop.sdrop_fwd_ex(dz, w0, m, scale_mode=sdrop.SCALE_ONE)
        if need_w0:
            dw0 = sdrop.sdrop_bwd_dw_ex(dz, h, m, scale_mode=sdrop.SCALE_ONE)
        if need_b0 and ctx.has_bias:
            db0 = sdrop.sdrop_bias_grad(dz, m)
        if need_w:
            dw = sdrop.sdrop_bwd_dw(x, dy, m)
        return dh, dw0, db0, dw, None, None, None, None, None, None


def sparse_act_block(h, w0, b0, w, p, act="relu", BM=128, BK=128, seed=0, rng_stream=0):
    """y = s (m' . act(h w0^T + b0)) w with a fresh block mask m' over the hidden activation.

    h [M, N0], w0 [K, N0] (one row per hidden feature), b0 fp32 [K] or None, w [K, N]: contiguous
    fp16 / bf16 GPU tensors; M % BM == 0, K % BK == 0, N0 % 8 == 0, N % 8 == 0.
    act: "relu", "gelu" (the exact form) or "gelu_tanh".
    """
    return _SparseActBlock.apply(h, w0, b0, w, float(p), int(BM), int(BK), int(seed), int(rng_stream), act)


def sparse_relu_block(h, w0, b0, w, p, BM=128, BK=128, seed=0, rng_stream=0):
    """sparse_act_block with a ReLU."""
    return sparse_act_block(h, w0, b0, w, p, "relu", BM, BK, seed, rng_stream)


class SparseDropLinear(torch.nn.Module):
    """Dropout(p) followed by Linear(K -> N), with the dropout block-structured and fused into the
    layer's three GEMMs (the layer substitution of Section 4).  The weight is stored [K, N] as in
    Section 3.1, or, with weight_layout="nk", [N, K] like torch.nn.Linear's (a state dict of such a layer then loads
    as it is).  In eval mode nothing is dropped (p = 0: all blocks kept, scale 1)."""

    def __init__(self, in_features, out_features, p=0.5, BM=128, BK=128, bias=True, seed=0,
                 dtype=torch.bfloat16, device="cuda", weight_layout="kn"):
        super().__init__()
        self.p, self.BM, self.BK, self.seed = float(p), int(BM), int(BK), int(seed)
        if weight_layout not in ("kn", "nk"):
            raise ValueError("weight_layout is 'kn' or 'nk'")
        self.weight_layout = weight_layout
        w = torch.empty(in_features, out_features, dtype=torch.float32)
        torch.nn.init.kaiming_uniform_(w.t(), a=5 ** 0.5)
        if weight_layout == "nk":
            w = w.t().contiguous()
        self.weight = torch.nn.Parameter(w.to(dtype=dtype, device=device))
        self.bias = torch.nn.Parameter(torch.zeros(out_features, dtype=dtype, device=device)) if bias else None
        self.calls = 0          # the mask's rng_stream: a new mask every forward call

    def forward(self, x):
        lead = x.shape[:-1]
        x2 = x.reshape(-1, x.shape[-1]).contiguous()
        p = self.p if self.training else 0.0
        y = sparsedrop_matmul(x2, self.weight, p, self.BM, self.BK, self.seed, self.calls, self.weight_layout)
        if self.training:
            self.calls += 1
        if self.bias is not None:
            y = y + self.bias
        return y.reshape(*lead, y.shape[-1])
