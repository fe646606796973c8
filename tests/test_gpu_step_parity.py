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


@pytest.mark.parametrize("name", ["tiny_bf16", "tiny_gqa"])
def test_captured_step_replays_match_direct_launches(name, dev, progress):
    """The step of a resident topology is replayed as a captured HIP graph.  Two engines on the
    same weights, one with the option off: every step (24 of them, alternating between a tree and
    its root-only sub-tree as planted candidates are accepted, the context growing, eager work -
    drafts read-outs, logits copies, synchronisations - between the replays) must give the same
    tokens, paths, drafts and logits bit for bit; a third run repeats the first after a new
    prefill on the same engine."""
    import numpy as np
    from tests.gpu_common import make_engine
    cfg = synth.CONFIGS[name]
    w = synth.make_weights(cfg, dev, with_bias=True)
    tree = synth.full_tree((3, 2, 2)[:cfg.k], "root")
    N = tree.n_nodes
    args = (list(tree.parent), list(tree.rank), list(tree.anchor))
    prompt = synth.prompt_tokens(cfg.seed + 5, 600, cfg.vocab).tolist()     # long enough for a fixed split count
    eng_g = make_engine(cfg, w, max_ctx=800, max_nodes=N, max_rows=64)
    eng_e = make_engine(cfg, w, max_ctx=800, max_nodes=N, max_rows=64)
    eng_e.set_option("graph", 0)
    eng_g.set_option("graph", 1)
    ref = make_engine(cfg, w, max_ctx=800, max_nodes=1, max_rows=8)
    ref.set_option("graph", 0)
    kids = [[c for c in range(N) if tree.parent[c] == v] for v in range(N)]

    def continuation(emitted, n):
        """`emitted` followed by what plain greedy decoding (root-only steps, launched directly)
        appends; recomputed when a near-tie made the tree step commit another token."""
        t = list(emitted[:-1]) + ref.prefill([prompt + list(emitted[:-1])])
        while len(t) < len(emitted) + n:
            t += ref.step([-1], [0], [0])[0]
        return t

    def run(eng, steps):
        emitted = eng.prefill([prompt])
        out = [list(emitted)]
        g = continuation(emitted, 8)
        for i in range(steps):
            if g[:len(emitted)] != emitted or len(g) < len(emitted) + cfg.k + 1:
                g = continuation(emitted, 8)
            if eng.drafts()[1][0] and i % 2 == 0:      # plant i/2 mod (k+1) true tokens along the last children
                cand = [(t + 3) % cfg.vocab for t in synth.prompt_tokens(i, N, cfg.vocab, stream=3).tolist()]
                v = 0
                for lvl in range((i // 2) % (cfg.k + 1)):
                    v = kids[v][-1]
                    cand[v] = g[len(emitted) + lvl]
                toks = eng.step_with_candidates(*args, [cand])[0]
            else:
                toks = eng.step(*args)[0]               # own drafts, or the root alone when there are none
            emitted += toks
            d, valid = eng.drafts()
            out.append((toks, eng.last_path()[0], d.tolist(), valid, eng.last_logits().copy()))
        return out

    a = run(eng_g, 24)
    b = run(eng_e, 24)
    assert eng_g.stat("graph_launches") >= 20 and eng_e.stat("graph_launches") == 0
    assert eng_g.stat("graph_captures") <= 6
    assert max(len(x[0]) for x in a[1:]) >= 2          # candidates were accepted
    assert any(x[4].shape[1] == 1 + cfg.k for x in a[1:])   # ... and root-only steps followed
    a2 = run(eng_g, 24)
    for x, y in ((a, b), (a, a2)):
        assert x[0] == y[0]
        for i, (p, q) in enumerate(zip(x[1:], y[1:])):
            assert p[0] == q[0] and p[1] == q[1] and p[2] == q[2] and p[3] == q[3], f"step {i}"
            assert np.array_equal(p[4], q[4]), f"step {i}: logits differ"
    progress(f"graph replays {name}: {eng_g.stat('graph_launches')} launches, {eng_g.stat('graph_captures')} captures")
