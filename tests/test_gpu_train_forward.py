"""Training-stage forward (Eq. 3-4) of the HIP library against the CPU oracle, through the C ABI."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2410_20488_amd import synth
from paper_2410_20488_amd.binding import FirpError
from tests.gpu_common import make_engine
from tests.helpers import cpu_weights, make_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name,layers,n,tol_logit,tol_kl", [
    ("tiny", None, 23, 1e-4, 1e-4), ("tiny", (1, 2, 3), 40, 1e-4, 1e-4), ("tiny", (0, 2, 4), 17, 1e-4, 1e-4),
    ("tiny_bf16", None, 64, 2e-2, 2e-3), ("tiny_bf16", (1, 2, 3), 37, 2e-2, 2e-3), ("tiny_gqa", None, 50, 2e-2, 2e-3),
    ("tiny_bf16", None, 100, 2e-2, 2e-3), ("tiny_bf16", (0, 1, 3), 128, 2e-2, 2e-3)])   # 200 and 256 rows
def test_train_forward_matches_oracle(name, layers, n, tol_logit, tol_kl, progress):
    """Every prediction step: all 2n rows of logits within the logit tolerance, every KL term
    within tol_kl of the largest term (the terms inherit the logits' error), the loss likewise."""
    cfg = synth.CONFIGS[name]
    if layers is not None:
        cfg = dataclasses.replace(cfg, firp_layers=layers[:cfg.k])
    w = synth.make_weights(cfg, DEV, with_bias=True)
    orc = make_oracle(cfg, cpu_weights(w), dtype=torch.float64)
    eng = make_engine(cfg, w, max_ctx=64, max_nodes=8, max_rows=2 * n)
    toks = synth.prompt_tokens(cfg.seed + 3, n, cfg.vocab).tolist()
    for step in range(1, cfg.k + 1):
        loss_ref, kl_ref, logits_ref = orc.train_forward(toks, step)
        loss, kl = eng.train_forward(toks, step)
        lg = eng.last_logits()[0]
        ref = logits_ref.double().numpy()
        assert lg.shape == ref.shape
        err = np.abs(lg.astype(np.float64) - ref).max() / ref.std()
        klr = kl_ref.double().numpy()
        kerr = np.abs(kl.astype(np.float64) - klr).max() / klr.max()
        progress(f"{name} step {step}: logit err {err:.2e}, kl err {kerr:.2e}, loss {loss:.4f} vs {loss_ref:.4f}")
        assert err <= tol_logit
        assert kerr <= tol_kl
        assert abs(loss - loss_ref) <= tol_kl * abs(loss_ref)


def test_train_forward_state_rules(progress):
    """It needs a context without sequences and leaves it so; decoding works afterwards."""
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg, DEV)
    eng = make_engine(cfg, w, max_ctx=64, max_nodes=8, max_rows=32)
    toks = synth.prompt_tokens(5, 12, cfg.vocab).tolist()
    loss0, _ = eng.train_forward(toks, 1)
    orc = make_oracle(cfg, cpu_weights(w), dtype=torch.float64)
    first = eng.prefill([toks])
    assert first == [orc.prefill(toks)]
    with pytest.raises(FirpError):
        eng.train_forward(toks, 1)                 # a sequence is alive
    tree = synth.full_tree((2, 2), "root")
    got = eng.step(list(tree.parent), list(tree.rank), list(tree.anchor))[0]
    assert got == orc.step(parent=list(tree.parent), rank=list(tree.rank), anchor=list(tree.anchor)).tokens
    eng.reset()
    loss1, _ = eng.train_forward(toks, 1)
    assert loss1 == loss0                          # same kernels, same order: bit-identical
    with pytest.raises(FirpError):
        eng.train_forward(toks, cfg.k + 1)
    with pytest.raises(FirpError):
        eng.train_forward(toks[:1], 1)
    with pytest.raises(FirpError):
        eng.train_forward(toks * 2, 1)             # 2n rows exceed max_rows
