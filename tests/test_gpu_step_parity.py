"""Whole-step parity of the HIP library against the CPU oracle, through the C ABI."""
import pytest
import torch

from paper_2410_20488_amd import synth
from tests.gpu_common import compare_cache, run_lockstep

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


def test_config1_tiny_fp32_chain_32_steps(dev, progress):
    """The small benchmark configuration: fp32, chain tree, 32 steps, exact tokens."""
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg, dev)
    rep, eng, orc = run_lockstep(cfg, w, synth.workload_tree("tiny"), prompt_len=64, n_steps=32, tol=1e-4,
                                 progress=progress)
    assert rep.steps == 32 and rep.tokens >= 32 and rep.tie_ambiguous == 0
    assert max(i for i, c in enumerate(rep.accepted_hist) if c) >= 3      # injection reached depth >= 2
    compare_cache(eng, orc, cfg)


@pytest.mark.parametrize("anchors", ["root", "all"])
def test_tiny_fp32_branching_tree_with_bias(dev, progress, anchors):
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg, dev, with_bias=True)
    tree = synth.full_tree((3, 2, 2), anchors)
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=37, n_steps=9, tol=1e-4, progress=progress)
    assert rep.tie_ambiguous == 0
    compare_cache(eng, orc, cfg)


def test_tiny_bf16_plain_kernels(dev, progress):
    cfg = synth.CONFIGS["tiny_bf16"]
    w = synth.make_weights(cfg, dev)
    rep, eng, orc = run_lockstep(cfg, w, synth.full_tree((3, 2), "root"), prompt_len=70, n_steps=9, tol=2e-2,
                                 gemm=0, progress=progress)
    compare_cache(eng, orc, cfg)


def test_tiny_gqa_random_tree(dev, progress):
    cfg = synth.CONFIGS["tiny_gqa"]
    w = synth.make_weights(cfg, dev, with_bias=True)
    tree = synth.random_tree(11, 13, 2, 4, 0.4)
    tree = synth.Tree(tree.parent, tree.rank, (1,) + tree.anchor[1:])
    run_lockstep(cfg, w, tree, prompt_len=150, n_steps=9, tol=2e-2, gemm=0, progress=progress)


def test_tiny_bf16_mfma_projection(dev, progress):
    cfg = synth.CONFIGS["tiny_bf16"]
    w = synth.make_weights(cfg, dev, with_bias=True)
    rep, eng, orc = run_lockstep(cfg, w, synth.full_tree((3, 2, 2), "all"), prompt_len=70, n_steps=9, tol=2e-2,
                                 gemm=1, progress=progress)
    compare_cache(eng, orc, cfg)


def test_tiny_gqa_mfma_random_tree(dev, progress):
    cfg = synth.CONFIGS["tiny_gqa"]
    w = synth.make_weights(cfg, dev, with_bias=True)
    tree = synth.random_tree(12, 17, 2, 4, 0.3)
    tree = synth.Tree(tree.parent, tree.rank, (1,) + tree.anchor[1:])
    run_lockstep(cfg, w, tree, prompt_len=150, n_steps=9, tol=2e-2, progress=progress)


@pytest.mark.parametrize("name,layers,gemm,tol", [("tiny", (1, 2, 3), None, 1e-4), ("tiny", (0, 2, 4), None, 1e-4),
                                                  ("tiny", (2, 2, 3), None, 1e-4), ("tiny_bf16", (1, 2, 3), 1, 2e-2),
                                                  ("tiny_bf16", (0, 3, 3), 1, 2e-2)])
@pytest.mark.parametrize("anchors", ["root", "all"])
def test_one_prediction_layer_per_step(dev, progress, name, layers, gemm, tol, anchors):
    """Pseudo hidden state i enters at its own layer t_i (Training stage; Setup uses three different
    layers): the step's row count grows through the stack."""
    import dataclasses
    cfg = dataclasses.replace(synth.CONFIGS[name], firp_layers=layers)
    w = synth.make_weights(cfg, dev, with_bias=True)
    tree = synth.full_tree((3, 2, 2), anchors)
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=41, n_steps=8, tol=tol, gemm=gemm, progress=progress)
    if cfg.dtype == "f32":
        assert rep.tie_ambiguous == 0
    compare_cache(eng, orc, cfg)


def test_7b_widths_4_layers_full_tree(dev, progress):
    """LLaMA-2-7B widths, 4 layers (the oracle finishes in seconds), the 41-node 4/3/2 tree."""
    cfg = synth.scaled_config(synth.CONFIGS["7b"], 4, 2)
    w = synth.make_weights(cfg, dev)
    rep, eng, orc = run_lockstep(cfg, w, synth.workload_tree("7b"), prompt_len=200, n_steps=6, tol=2e-2,
                                 progress=progress)
    progress(f"7b/4 layers: max logit err {rep.max_logit_err:.3e}, ties {rep.tie_ambiguous}")
    compare_cache(eng, orc, cfg)


@pytest.mark.parametrize("name,seed", [("tiny_bf16", 3), ("tiny_gqa", 5), ("tiny", 7)])
def test_small_model_steps_are_bit_repeatable(dev, progress, name, seed):
    """Prefill and four steps with an irregular tree (two sequences of different length), forty times
    on one engine: identical tokens and identical logits, bit for bit, every time."""
    import numpy as np
    from tests.gpu_common import make_engine
    cfg = synth.CONFIGS[name]
    w = synth.make_weights(cfg, dev, with_bias=True)
    tree = synth.random_tree(seed, 19, cfg.k, 4, 0.6)
    n_rows = tree.n_nodes + cfg.k * sum(tree.anchor)
    prompts = [synth.prompt_tokens(seed, 150, cfg.vocab).tolist(), synth.prompt_tokens(seed, 9, cfg.vocab, stream=1).tolist()]
    args = (list(tree.parent), list(tree.rank), list(tree.anchor))
    eng = make_engine(cfg, w, max_ctx=220, max_batch=2, max_nodes=tree.n_nodes, max_rows=n_rows, b_max=8)
    ref, bad = None, 0
    for it in range(40):
        outs = [np.array(eng.prefill(prompts))]
        for _ in range(4):
            toks = eng.step(*args)
            outs.append(np.array([t + [-1] * (cfg.k + 1 - len(t)) for t in toks]))
            outs.append(eng.last_logits().copy())
        if ref is None:
            ref = outs
        elif not all(np.array_equal(a, b) for a, b in zip(outs, ref)):
            bad += 1
    progress(f"repeatability {name}: {bad} of 39 runs differ from the first")
    assert bad == 0
