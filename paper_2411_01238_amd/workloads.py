"""Seeded synthetic inputs for SparseDrop's hot path.

This module holds the five workload shapes and their input recipes and nothing
of the method's arithmetic: no mask rule, no product, no scaling.  Both the
HIP path's tests/benchmark and the CPU oracle's tests draw their inputs here,
so the two sides see identical bits.

The paper (arxiv 2411.01238) trains on MNIST, Fashion-MNIST, CIFAR-10 and
Shakespeare (Section 4.1); none of that data is used.  The tensors below are
synthetic stand-ins with the shapes the paper's layers have (hidden size 1024,
128x128 blocks, 16-bit mixed precision; Sections 4 and A) and simple value
distributions.  Every tensor is drawn on the CPU in float64 from a
``torch.Generator`` with a fixed seed and then rounded once to the 16-bit
storage type, so its float64 widening is exact.
"""
from dataclasses import dataclass, field
from typing import Tuple

import torch

SEED_X, SEED_W, SEED_DY = 1, 2, 3


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    K: int
    N: int
    BM: int
    BK: int
    dtype: str                      # "f16" or "bf16"
    ps: Tuple[float, ...]           # dropout rates the workload is run at
    x_dist: str                     # "normal" | "uniform" | "gelu"
    w_std: float
    layers: int = 1
    mask_seed: int = 0

    @property
    def MB(self):
        return self.M // self.BM

    @property
    def KB(self):
        return self.K // self.BK

    @property
    def torch_dtype(self):
        return {"f16": torch.float16, "bf16": torch.bfloat16}[self.dtype]


WORKLOADS = {
    # small case the oracle finishes in well under a second
    "tiny": Workload("tiny", 256, 256, 256, 64, 64, "f16", (0.5,), "normal", 1.0),
    # the headline sweep
    "square4096": Workload("square4096", 4096, 4096, 4096, 128, 128, "bf16",
                           (0.0, 0.1, 0.3, 0.5, 0.7), "normal", 1.0),
    # one layer of a 4-layer MLP classifier, batch 8192, hidden 1024
    "mlp": Workload("mlp", 8192, 1024, 1024, 64, 64, "f16", (0.1, 0.5), "uniform",
                    1.0 / 32.0, layers=4),
    # transformer FFN down-projection after the activation
    "ffn_down": Workload("ffn_down", 16384, 3072, 768, 128, 64, "bf16", (0.1,), "gelu", 0.02),
    # large skinny, HBM-pressure case
    "skinny": Workload("skinny", 65536, 4096, 1024, 128, 128, "bf16", (0.3,), "normal",
                       1.0 / 64.0),
}


def _draw(shape, seed, dist, std, dtype):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    rows, cols = shape
    out = torch.empty(shape, dtype=dtype)
    # drawn in row chunks so that the float64 staging buffer stays small
    step = max(1, (1 << 24) // cols)
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        if dist == "uniform":
            z = torch.rand((r1 - r0, cols), generator=g, dtype=torch.float64) * 2.0 - 1.0
        else:
            z = torch.randn((r1 - r0, cols), generator=g, dtype=torch.float64)
            if dist == "gelu":
                z = 0.5 * z * (1.0 + torch.special.erf(z * 0.7071067811865476))
        out[r0:r1] = (z * std).to(dtype)
    return out


def make_inputs(w, layer=0, M=None):
    """(X[M,K], W[K,N], dY[M,N]) as CPU tensors of the workload's 16-bit type.

    ``layer`` offsets the seeds (by 10 per layer) for the stacked-layer
    workload.  ``M`` may shrink the row count (a multiple of BM) for reduced
    copies of a workload; the recipe is otherwise unchanged.
    """
    M = w.M if M is None else M
    assert M % w.BM == 0
    dt = w.torch_dtype
    off = 10 * layer
    X = _draw((M, w.K), SEED_X + off, w.x_dist, 1.0, dt)
    W = _draw((w.K, w.N), SEED_W + off, "normal", w.w_std, dt)
    dY = _draw((M, w.N), SEED_DY + off, "normal", 1.0, dt)
    return X, W, dY


def make_custom(M, K, N, dtype, seed=0, w_std=1.0):
    """Plain N(0,1) / N(0,w_std^2) inputs of an arbitrary shape (edge-case tests)."""
    dt = {"f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    X = _draw((M, K), 100 + seed, "normal", 1.0, dt)
    W = _draw((K, N), 200 + seed, "normal", w_std, dt)
    dY = _draw((M, N), 300 + seed, "normal", 1.0, dt)
    return X, W, dY
