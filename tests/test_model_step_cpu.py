"""CPU checks of the whole-model harness (arxiv 2411.01238, Section 4.1 layer substitution): the
variants that need no GPU must agree where the mathematics says so.  The SparseDrop variant itself
runs in the HIP kernels only and is checked in test_gpu_model_step.py."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd import model_step as ms

CFG = {
    "mlp": dict(in_dim=256, hidden=256, n_hidden=1, n_out=10),
    "vit": dict(image=16, patch=2, d=128, n_layers=1, n_head=2, n_out=10),
    "gpt": dict(vocab=65, context=32, d=128, n_layers=1, n_head=2),
}
BATCH = {"mlp": 256, "vit": 4, "gpt": 8}       # 256 rows in every substituted layer


def _batch(name):
    shape = {k: v for k, v in CFG[name].items() if k in ("in_dim", "n_out", "image", "context", "vocab")}
    return ms.synthetic_batch(name, seed=1, device="cpu", dtype=torch.float64, batch=BATCH[name], **shape)


def _pair(name, kind_a, kind_b, p, keep_fn=None):
    torch.manual_seed(0)
    a = ms.MODELS[name](kind_a, p, dtype=torch.float64, device="cpu", keep_fn=keep_fn, **CFG[name])
    b = ms.MODELS[name](kind_b, p, dtype=torch.float64, device="cpu", keep_fn=keep_fn, **CFG[name])
    b.load_state_dict(a.state_dict())
    return a.train(), b.train()


@pytest.mark.parametrize("name", ["mlp", "vit", "gpt"])
def test_block_dropout_with_everything_kept_is_the_dense_model(name):
    a, b = _pair(name, "dense", "block_dropout_dense", 0.0, keep_fn=lambda MB, KB, p, seed, call: np.ones((MB, KB)))
    batch = _batch(name)
    la, lb = a.loss(batch), b.loss(batch)
    la.backward(); lb.backward()
    assert abs(la.item() - lb.item()) <= 1e-12 * abs(la.item())
    for (n, x), (_, y) in zip(a.named_parameters(), b.named_parameters()):
        assert torch.allclose(x.grad, y.grad, rtol=1e-10, atol=1e-12), n


@pytest.mark.parametrize("name", ["mlp", "vit", "gpt"])
def test_each_layer_and_step_asks_for_its_own_mask(name):
    calls = []

    def keep_fn(MB, KB, p, seed, call):
        calls.append((seed, call))
        return np.asarray(orc.mask(MB, KB, p, seed, call))

    torch.manual_seed(0)
    m = ms.MODELS[name]("block_dropout_dense", 0.5, dtype=torch.float64, device="cpu", keep_fn=keep_fn, **CFG[name]).train()
    batch = _batch(name)
    m.loss(batch).backward()
    first = list(calls)
    m.loss(batch).backward()
    second = calls[len(first):]
    assert len(set(first)) == len(first)                         # one (seed, call) per substituted layer
    assert [s for s, _ in first] == [s for s, _ in second]      # the same layers, in the same order
    assert all(c == 0 for _, c in first) and all(c == 1 for _, c in second)
    # evaluation draws nothing new: p = 0 there, and the call numbers stand still
    m.eval()
    with torch.no_grad():
        m.loss(batch)
    assert [c for _, c in calls[len(first) + len(second):]] == [2] * len(first)
    m.train()
    m.loss(batch)
    assert calls[-1][1] == 2


def test_dropout_rate_zero_makes_the_variants_equal():
    a, b = _pair("mlp", "dense", "dropout_dense", 0.0)
    batch = _batch("mlp")
    assert a.loss(batch).item() == b.loss(batch).item()


def test_unknown_kinds_are_refused():
    with pytest.raises(ValueError):
        ms.Linear("sparse", 128, 128, 0.5, 0, torch.float64, "cpu")
    with pytest.raises(ValueError):
        ms.synthetic_batch("resnet", device="cpu")
