"""Whole models with substituted linear layers (arxiv 2411.01238, Section 4.1 and 4.3): the SparseDrop
variant must compute what the same model computes in float64 on the CPU when every substituted layer
applies, as a dense element mask, the block mask that the ORACLE draws for that layer's seed and call
number.  This checks the wiring (one mask per layer and per step, the same mask in forward and
backward, scale 1/(1-p)); the kernels themselves are checked element by element elsewhere.

The 16-bit model rounds every activation, the reference none: the tolerance is that of a chain of
fp16 roundings (a wrong mask, seed or scale gives errors of order one)."""
import numpy as np
import pytest
import torch

from oracle import sdrop_oracle as orc
from paper_2411_01238_amd import model_step as ms
from _util import errors

pytestmark = pytest.mark.gpu

SMALL = {
    "mlp": dict(in_dim=256, hidden=512, n_hidden=1, n_out=10),
    "vit": dict(image=16, patch=2, d=384, n_layers=1, n_head=3, n_out=10),
    "gpt": dict(vocab=65, context=64, d=384, n_layers=2, n_head=3),
}
BATCH = {"mlp": 384, "vit": 8, "gpt": 8}     # 384, 512 and 512 rows in the substituted layers


@pytest.mark.parametrize("name", ["mlp", "vit", "gpt"])
@pytest.mark.parametrize("p", [0.5, 0.2])
def test_sparsedrop_model_matches_float64_model_with_the_oracles_masks(name, p):
    print("model", name, p, flush=True)
    torch.manual_seed(3)
    cfg = SMALL[name]
    model = ms.MODELS[name]("sparsedrop", p, dtype=torch.float16, **cfg)
    ref = ms.MODELS[name]("block_dropout_dense", p, dtype=torch.float64, device="cpu",
                          keep_fn=lambda MB, KB, p_, seed, call: np.asarray(orc.mask(MB, KB, p_, seed, call)), **cfg)
    ref.load_state_dict({k: v.detach().cpu().double() for k, v in model.state_dict().items()})
    shape = {k: v for k, v in cfg.items() if k in ("in_dim", "n_out", "image", "context", "vocab")}
    model.train(); ref.train()
    for step in range(2):                        # the second step must use each layer's next mask
        batch = ms.synthetic_batch(name, seed=step, dtype=torch.float16, batch=BATCH[name], **shape)
        rbatch = tuple(t.cpu().double() if t.is_floating_point() else t.cpu() for t in batch)
        for mdl in (model, ref):
            for prm in mdl.parameters():
                prm.grad = None
        loss = model.loss(batch); loss.backward()
        rloss = ref.loss(rbatch); rloss.backward()
        torch.cuda.synchronize()
        assert abs(loss.item() - rloss.item()) <= 2e-2 * abs(rloss.item()), (step, loss.item(), rloss.item())
        for (n, prm), (_, rprm) in zip(model.named_parameters(), ref.named_parameters()):
            if rprm.grad is None:
                assert prm.grad is None, n
                continue
            got, want = prm.grad.double().cpu().numpy(), rprm.grad.numpy()
            assert np.all(np.isfinite(got)), n
            fro, _ = errors(got, want)
            assert fro <= 3e-2, "step %d, %s: relative Frobenius error %.3e" % (step, n, fro)


def test_eval_mode_drops_nothing_and_variants_agree():
    torch.manual_seed(4)
    cfg = SMALL["mlp"]
    a = ms.MLP("sparsedrop", 0.5, dtype=torch.float16, **cfg).eval()
    b = ms.MLP("dense", 0.0, dtype=torch.float16, **cfg).eval()
    b.load_state_dict(a.state_dict())
    x, _ = ms.synthetic_batch("mlp", seed=1, dtype=torch.float16, batch=256, in_dim=256)
    with torch.no_grad():
        fro, _ = errors(a(x).double().cpu().numpy(), b(x).double().cpu().numpy())
    assert fro <= 2e-3, fro
