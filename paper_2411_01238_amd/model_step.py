"""Forward + backward time of whole models whose linear layers are substituted.

arxiv 2411.01238, Section 4.1 (layer substitution) and Section 4.3 ("Real-world throughput"):
every linear layer of a model is one of

    dense            x W                         (no dropout, no bias: Section 3.1)
    dropout_dense    dropout(x, p) W             (element-wise dropout from torch, then a dense GEMM)
    sparsedrop       s (x . m') W                (eq. (1)-(3) in libsdrop's kernels, one block mask per call)

and the time of one forward + backward pass is measured over the dropout rate.  The models follow
the configurations of the paper's appendix: an MLP (input, two hidden and output layers, width
1024, ReLU, batch 1024 of 32 x 32 images), a two-layer ViT (2 x 2 patches of a 32 x 32 image = 256
tokens, width 1024, 8 heads, batch 64) and a four-layer GPT (context 128, width 1024, 8 heads,
batch 32, character vocabulary).  Batches are synthetic (random pixels / tokens and labels): the
measurement is of time, not of accuracy.

Everything outside the substituted layers (layer norms, attention, GELU, embeddings, the loss) is
plain PyTorch and the same in the three variants.  Layers whose input is narrower than a mask
block (the ViT's patch embedding, 4 features) or has fewer rows than one (its classifier on the
pooled vector) stay dense in every variant.  Output widths are padded to a multiple of 8 (10 -> 16
classes, 65 -> 72 characters); the loss reads the unpadded columns.

    python -m paper_2411_01238_amd.model_step --model all --p 0 0.1 0.2 0.3 0.4 0.5 0.6 0.7
"""
import argparse
import json
import math

import torch
import torch.nn.functional as F

from .autograd import sparsedrop_matmul

KINDS = ("dense", "dropout_dense", "sparsedrop")
BLOCK = 128                     # the paper's experiments use 128 x 128 mask blocks throughout


def _pad8(n):
    return (n + 7) // 8 * 8


class Linear(torch.nn.Module):
    """One substituted layer: x [.., K] -> [.., N] with the weight stored [K, N].

    `kind` is one of KINDS, or "block_dropout_dense": the block mask applied as a dense element
    mask in plain torch, with the keep flags of each call taken from `keep_fn(MB, KB, p, seed,
    rng_stream)`: for checks of the wiring against a mask source of the caller's choice.
    A sparsedrop layer draws mask number `calls` of its own seed, so that a model's layers and
    steps all see different masks.
    """

    def __init__(self, kind, K, N, p, seed, dtype, device, keep_fn=None):
        super().__init__()
        if kind not in KINDS + ("block_dropout_dense",):
            raise ValueError(f"unknown layer kind {kind!r}")
        self.kind, self.p, self.seed, self.keep_fn, self.calls = kind, float(p), int(seed), keep_fn, 0
        g = torch.Generator(device="cpu")
        g.manual_seed(1000 + seed)
        w = (torch.rand(K, N, generator=g, dtype=torch.float64) * 2 - 1) / math.sqrt(K)
        self.weight = torch.nn.Parameter(w.to(dtype=dtype, device=device))

    def forward(self, x):
        lead, K = x.shape[:-1], x.shape[-1]
        x2 = x.reshape(-1, K)
        p = self.p if self.training else 0.0
        if self.kind == "sparsedrop":
            y = sparsedrop_matmul(x2.contiguous(), self.weight, p, BLOCK, BLOCK, self.seed, self.calls)
        elif self.kind == "block_dropout_dense":
            M = x2.shape[0]
            keep = torch.as_tensor(self.keep_fn(M // BLOCK, K // BLOCK, p, self.seed, self.calls))
            m = keep.to(device=x2.device, dtype=x2.dtype).repeat_interleave(BLOCK, 0).repeat_interleave(BLOCK, 1)
            y = ((x2 * m) @ self.weight) * (1.0 / (1.0 - p) if p < 1.0 else 0.0)
        else:
            if self.kind == "dropout_dense" and p > 0.0:
                x2 = F.dropout(x2, p, training=True)
            y = x2 @ self.weight
        if self.training:
            self.calls += 1
        return y.reshape(*lead, y.shape[-1])


class MLP(torch.nn.Module):
    """Input layer, `n_hidden` hidden layers and an output layer, ReLU between them (Section 4.2, MLP)."""

    def __init__(self, kind, p, in_dim=1024, hidden=1024, n_hidden=2, n_out=10, dtype=torch.bfloat16,
                 device="cuda", keep_fn=None):
        super().__init__()
        dims = [in_dim] + [hidden] * (n_hidden + 1) + [_pad8(n_out)]
        self.n_out = n_out
        self.layers = torch.nn.ModuleList(
            Linear(kind, dims[i], dims[i + 1], p, i, dtype, device, keep_fn) for i in range(len(dims) - 1))

    def forward(self, x):
        for i, layer in enumerate(self.layers):
            x = layer(x if i == 0 else F.relu(x))
        return x[..., :self.n_out]

    def loss(self, batch):
        x, labels = batch
        return F.cross_entropy(self(x).float(), labels)


class Block(torch.nn.Module):
    """Pre-norm transformer block; its four linear layers are the substituted ones."""

    def __init__(self, kind, p, d, n_head, causal, seed, dtype, device, keep_fn):
        super().__init__()
        self.n_head, self.causal = n_head, causal
        self.ln1 = torch.nn.LayerNorm(d, dtype=dtype, device=device)
        self.ln2 = torch.nn.LayerNorm(d, dtype=dtype, device=device)
        self.qkv = Linear(kind, d, 3 * d, p, seed, dtype, device, keep_fn)
        self.proj = Linear(kind, d, d, p, seed + 1, dtype, device, keep_fn)
        self.fc = Linear(kind, d, 4 * d, p, seed + 2, dtype, device, keep_fn)
        self.fc2 = Linear(kind, 4 * d, d, p, seed + 3, dtype, device, keep_fn)

    def forward(self, x):
        B, T, d = x.shape
        q, k, v = self.qkv(self.ln1(x)).view(B, T, 3, self.n_head, d // self.n_head).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(q, k, v, is_causal=self.causal)
        x = x + self.proj(a.transpose(1, 2).reshape(B, T, d))
        return x + self.fc2(F.gelu(self.fc(self.ln2(x))))


class ViT(torch.nn.Module):
    """Patches of a one-channel image as tokens, transformer blocks, mean pooling, classifier (Section 4.2, ViT)."""

    def __init__(self, kind, p, image=32, patch=2, d=1024, n_layers=2, n_head=8, n_out=10, dtype=torch.bfloat16,
                 device="cuda", keep_fn=None):
        super().__init__()
        self.patch, self.n_tokens = patch, (image // patch) ** 2
        self.embed = torch.nn.Linear(patch * patch, d, dtype=dtype, device=device)
        self.pos = torch.nn.Parameter(torch.zeros(self.n_tokens, d, dtype=dtype, device=device))
        self.blocks = torch.nn.ModuleList(
            Block(kind, p, d, n_head, False, 10 * i, dtype, device, keep_fn) for i in range(n_layers))
        self.ln = torch.nn.LayerNorm(d, dtype=dtype, device=device)
        self.head = torch.nn.Linear(d, n_out, dtype=dtype, device=device)

    def forward(self, img):
        B, s = img.shape[0], self.patch
        x = img.unfold(1, s, s).unfold(2, s, s).reshape(B, self.n_tokens, s * s)
        x = self.embed(x) + self.pos
        for b in self.blocks:
            x = b(x)
        return self.head(self.ln(x).mean(dim=1))

    def loss(self, batch):
        img, labels = batch
        return F.cross_entropy(self(img).float(), labels)


class GPT(torch.nn.Module):
    """Decoder-only transformer over characters; the output layer is a substituted one too (Section 4.2, language modelling)."""

    def __init__(self, kind, p, vocab=65, context=128, d=1024, n_layers=4, n_head=8, dtype=torch.bfloat16,
                 device="cuda", keep_fn=None):
        super().__init__()
        self.vocab = vocab
        self.tok = torch.nn.Embedding(vocab, d, dtype=dtype, device=device)
        self.pos = torch.nn.Parameter(torch.zeros(context, d, dtype=dtype, device=device))
        self.blocks = torch.nn.ModuleList(
            Block(kind, p, d, n_head, True, 10 * i, dtype, device, keep_fn) for i in range(n_layers))
        self.ln = torch.nn.LayerNorm(d, dtype=dtype, device=device)
        self.lm_head = Linear(kind, d, _pad8(vocab), p, 10 * n_layers, dtype, device, keep_fn)

    def forward(self, tokens):
        x = self.tok(tokens) + self.pos[:tokens.shape[1]]
        for b in self.blocks:
            x = b(x)
        return self.lm_head(self.ln(x))[..., :self.vocab]

    def loss(self, batch):
        tokens, targets = batch
        return F.cross_entropy(self(tokens).float().reshape(-1, self.vocab), targets.reshape(-1))


def synthetic_batch(name, seed=0, device="cuda", dtype=torch.bfloat16, batch=None, **shape):
    """Random pixels in [0, 1) with random labels, or random characters with random next characters."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    if name == "mlp":
        B, n = batch or 1024, shape.get("in_dim", 1024)
        return (torch.rand(B, n, generator=g).to(device=device, dtype=dtype),
                torch.randint(0, shape.get("n_out", 10), (B,), generator=g).to(device))
    if name == "vit":
        B, s = batch or 64, shape.get("image", 32)
        return (torch.rand(B, s, s, generator=g).to(device=device, dtype=dtype),
                torch.randint(0, shape.get("n_out", 10), (B,), generator=g).to(device))
    if name == "gpt":
        B, T, V = batch or 32, shape.get("context", 128), shape.get("vocab", 65)
        return (torch.randint(0, V, (B, T), generator=g).to(device), torch.randint(0, V, (B, T), generator=g).to(device))
    raise ValueError(f"unknown model {name!r}")


MODELS = {"mlp": MLP, "vit": ViT, "gpt": GPT}


def time_step(model, batch, steps=20, warmup=5):
    """Milliseconds of one forward + backward pass (training mode), averaged over `steps`, as issued
    from Python: at the paper's batch sizes the MLP and GPT passes are bound by the host issuing
    launches on this chip (every variant alike), the ViT pass by the GPU."""
    model.train()

    def step():
        for prm in model.parameters():
            prm.grad = None
        model.loss(batch).backward()

    for _ in range(warmup):
        step()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(steps):
        step()
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / steps


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--model", default="all", choices=tuple(MODELS) + ("all",))
    ap.add_argument("--p", type=float, nargs="+", default=[0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7])
    ap.add_argument("--dtype", default="bf16", choices=("bf16", "f16"))
    ap.add_argument("--batch-scale", type=int, default=1,
                    help="multiply the paper's batch sizes (1024 / 64 / 32) by this: larger batches are bound by the GPU, not the host")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        raise SystemExit("model_step needs a GPU: the substituted layers run in libsdrop's kernels only")
    dtype = torch.bfloat16 if a.dtype == "bf16" else torch.float16
    for name in (tuple(MODELS) if a.model == "all" else (a.model,)):
        batch = synthetic_batch(name, dtype=dtype, batch={"mlp": 1024, "vit": 64, "gpt": 32}[name] * a.batch_scale)
        ms = time_step(MODELS[name]("dense", 0.0, dtype=dtype), batch, a.steps, a.warmup)
        print(json.dumps({"model": name, "batch": batch[0].shape[0], "layer": "dense", "p": None, "ms_fwd_bwd": round(ms, 4)}), flush=True)
        for p in a.p:
            row = {"model": name, "batch": batch[0].shape[0], "p": p}
            for kind in ("dropout_dense", "sparsedrop"):
                row[kind + "_ms_fwd_bwd"] = round(time_step(MODELS[name](kind, p, dtype=dtype), batch, a.steps, a.warmup), 4)
            row["speedup"] = round(row["dropout_dense_ms_fwd_bwd"] / row["sparsedrop_ms_fwd_bwd"], 3)
            print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()
