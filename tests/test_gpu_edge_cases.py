"""Edge cases of the step through the C ABI: several sequences, degenerate FIRP settings
(k = 0, l = 0, l = L), every node an anchor with more than 128 rows, a long context, the largest
k and b, a one-token prompt, a context that fills up."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2410_20488_amd import synth
from tests.gpu_common import compare_cache, make_engine, run_lockstep, run_lockstep_batch
from tests.helpers import cpu_weights, make_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name,tol", [("tiny", 1e-4), ("tiny_bf16", 2e-2)])
def test_two_sequences_with_different_prompts(progress, name, tol):
    """Independent sequences share weights and topology, have their own cache length, drafts and
    path; a sequence without drafts rides along with 'no candidate' tokens and must return what
    its own root-only step returns.  (bf16: the MFMA kernels, whose prefill runs every sequence
    as a batch of one at its own cache offset.)"""
    cfg = synth.CONFIGS[name]
    w = synth.make_weights(cfg, DEV, with_bias=True)
    tree = synth.full_tree((3, 2), "root")
    rep, eng, orcs = run_lockstep_batch(cfg, w, tree, prompt_lens=[70, 23], n_steps=8, tol=tol, max_rows=32,
                                        progress=progress)
    assert rep.steps == 8
    assert sum(rep.accepted_hist[2:]) > 0        # planted continuations were accepted
    if name == "tiny":
        assert rep.tie_ambiguous == 0


@pytest.mark.parametrize("k,layer", [(0, 2), (3, 0), (3, 4), (1, 3)])
def test_degenerate_firp_settings(k, layer, progress):
    """k = 0 is plain greedy decoding; l = 0 maps the embeddings; l = L sends the mapped states
    straight to the final norm and lm-head."""
    cfg = dataclasses.replace(synth.CONFIGS["tiny"], k=k, firp_layer=layer)
    w = synth.make_weights(cfg, DEV, with_bias=True)
    tree = synth.full_tree((2, 2, 2)[:max(k, 1)], "all") if k else synth.chain_tree(3, "none")
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=19, n_steps=7, tol=1e-4, progress=progress, max_rows=64)
    assert rep.tie_ambiguous == 0
    if k == 0:
        # the whole run is ordinary greedy decoding, token for token
        ref = make_oracle(cfg, cpu_weights(w), dtype=torch.float64)
        prompt = synth.prompt_tokens(cfg.seed, 19, cfg.vocab).tolist()
        want = ref.greedy(prompt, 4)
        eng2 = make_engine(cfg, w, max_ctx=64, max_nodes=4, max_rows=8)
        got = eng2.prefill([prompt])
        while len(got) < 4:
            got += eng2.step(list(tree.parent), list(tree.rank), list(tree.anchor))[0]
        assert got[:4] == want
    compare_cache(eng, orc, cfg)


def test_every_node_an_anchor_256_rows(progress):
    """The paper-complete setting: all 64 nodes carry k = 3 pseudo rows, 256 rows above the
    FIRP layer (two row blocks of the projection kernel), at LLaMA-2-7B widths."""
    cfg = synth.scaled_config(synth.CONFIGS["7b"], 2, 1)
    w = synth.make_weights(cfg, DEV)
    tree = synth.workload_tree("13b", "all")
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=96, n_steps=4, tol=2e-2, progress=progress,
                                 max_rows=256)
    progress(f"A=all: max logit err {rep.max_logit_err:.2e}, ties {rep.tie_ambiguous}, hist {rep.accepted_hist}")
    assert max(i for i, c in enumerate(rep.accepted_hist) if c) >= 2


def test_long_context_7b_widths(progress):
    """A 4k-token context (the long-context workload at reduced depth): many cache splits,
    position ids in the thousands."""
    cfg = synth.scaled_config(synth.CONFIGS["7b"], 2, 1)
    w = synth.make_weights(cfg, DEV)
    tree = synth.workload_tree("13b", "root")
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=4100, n_steps=3, tol=2e-2, progress=progress)
    progress(f"long ctx: max logit err {rep.max_logit_err:.2e}")
    compare_cache(eng, orc, cfg)


def test_maximum_steps_and_candidates(progress):
    """The largest k and b the library takes: 8 prediction steps, top-16 candidates, a tree eight
    levels deep (a chain plus branching near the root), with per-step layers on top."""
    cfg = dataclasses.replace(synth.CONFIGS["tiny"], k=8, firp_layers=(0, 1, 1, 2, 2, 3, 3, 4))
    w = synth.make_weights(cfg, DEV, with_bias=True)
    paths = [()] + [tuple([0] * j) for j in range(1, 9)] + [(r,) for r in range(1, 16)] + [(15, 15), (3, 7, 9)]
    paths += [(3, 7)]
    paths = sorted(set(paths), key=lambda p: (len(p), p))
    index = {p: i for i, p in enumerate(paths)}
    parent = [-1] + [index[p[:-1]] for p in paths[1:]]
    rank = [0] + [p[-1] for p in paths[1:]]
    tree = synth.Tree(tuple(parent), tuple(rank), tuple([1] + [0] * (len(paths) - 1)))
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=30, n_steps=8, tol=1e-4, progress=progress, b_max=16,
                                 max_rows=64)
    assert rep.tie_ambiguous == 0
    assert max(i for i, c in enumerate(rep.accepted_hist) if c) >= 3
    compare_cache(eng, orc, cfg)


def test_one_token_prompt_and_full_context(progress):
    """A prompt of one token (nothing to prefill, the root-only step runs on an empty cache), then
    decoding until the context is full: the step that would not fit is refused with a capacity
    error, nothing is enqueued, and the context stays usable after a reset."""
    from paper_2410_20488_amd.binding import FirpError
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg, DEV)
    orc = make_oracle(cfg, cpu_weights(w), dtype=torch.float64)
    eng = make_engine(cfg, w, max_ctx=12, max_nodes=4, max_rows=16)
    tree = synth.chain_tree(3, "root")
    args = dict(parent=list(tree.parent), rank=list(tree.rank), anchor=list(tree.anchor))
    prompt = [17]
    assert eng.prefill([prompt]) == [orc.prefill(prompt)]
    assert eng.ctx_len() == [1] and orc.p0 == 1      # the root-only step committed the prompt's token
    emitted = 0
    with pytest.raises(FirpError) as e:
        for _ in range(40):
            want = orc.step(**args).tokens if orc.p0 + 4 <= 12 else None
            got = eng.step(args["parent"], args["rank"], args["anchor"])[0]
            assert want is not None and got == want
            emitted += len(got)
    assert "max_ctx" in str(e.value) and emitted >= 8
    full = eng.ctx_len()[0]
    assert full + 4 > 12                       # no room for a root plus three levels
    eng.reset()
    assert eng.prefill([prompt]) == [orc.fork().prefill(prompt)]


@pytest.mark.parametrize("name,tol", [("tiny", 1e-4), ("tiny_bf16", 2e-2)])
def test_full_tree_and_root_only_tree_alternate_without_uploads(progress, name, tol):
    """With the root as the only anchor, a step that accepts a candidate ends on a node without
    pseudo rows, so the next step has no drafts and runs on the root alone; the one after runs
    the full tree again.  Twenty steps of that alternation in lockstep with the oracle; the
    library keeps both topologies on the device, so the whole run uploads exactly two."""
    cfg = synth.CONFIGS[name]
    w = synth.make_weights(cfg, DEV, with_bias=True)
    tree = synth.full_tree((3, 2), "root")
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=40, n_steps=20, tol=tol, progress=progress, max_rows=32)
    assert rep.steps == 20 and sum(rep.accepted_hist[2:]) >= 4      # planted continuations were accepted
    assert eng.stat("topo_uploads") == 2, eng.stat("topo_uploads")
    if name == "tiny":
        assert rep.tie_ambiguous == 0
    compare_cache(eng, orc, cfg)


def test_more_topologies_than_the_library_keeps(progress):
    """Six different trees in rotation on one engine (the library keeps four): every step is
    checked against the oracle, whatever slot its tables were uploaded to or evicted from."""
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg, DEV, with_bias=True)
    orc = make_oracle(cfg, cpu_weights(w), dtype=torch.float64)
    eng = make_engine(cfg, w, max_ctx=200, max_nodes=16, max_rows=64)
    trees = [synth.full_tree((3, 2), "root"), synth.full_tree((2, 2, 2), "all"), synth.chain_tree(3, "root"),
             synth.random_tree(4, 12, 3, 4, 0.5), synth.full_tree((4,), "all"), synth.random_tree(9, 9, 2, 3, 1.0)]
    trees = [synth.Tree(t.parent, t.rank, (1,) + tuple(t.anchor[1:])) for t in trees]   # root an anchor: drafts stay valid
    prompt = synth.prompt_tokens(cfg.seed, 25, cfg.vocab).tolist()
    assert eng.prefill([prompt]) == [orc.prefill(prompt)]
    for step in range(18):
        t = trees[step % len(trees)]
        args = dict(parent=list(t.parent), rank=list(t.rank), anchor=list(t.anchor))
        r = orc.step(**args)
        got = eng.step(args["parent"], args["rank"], args["anchor"])[0]
        assert got == r.tokens and eng.last_path()[0] == r.path, f"step {step}"
        lg = eng.last_logits()[0]
        ref = r.logits.numpy()
        assert lg.shape == ref.shape and np.abs(lg - ref).max() / ref.std() < 1e-4, f"step {step}"
        if r.drafts is not None:
            assert eng.drafts()[0][0].tolist() == r.drafts
    # 1 (the prefill's root-only step) + 6 first uses + the re-uploads of evicted ones
    assert eng.stat("topo_uploads") >= 7


@pytest.mark.parametrize("name", ["tiny", "tiny_bf16"])
def test_steps_without_kept_logits(name):
    """By default a step leaves no logits in memory (it needs the greedy token of every node and
    the top-b ids of the pseudo rows only): tokens, paths, drafts and cache lengths must be those
    of an engine that keeps them, and the logits read-out must refuse."""
    from paper_2410_20488_amd.binding import FirpError
    cfg = synth.CONFIGS[name]
    w = synth.make_weights(cfg, DEV, with_bias=True)
    tree = synth.full_tree((3, 2), "all")
    args = (list(tree.parent), list(tree.rank), list(tree.anchor))
    prompt = synth.prompt_tokens(cfg.seed + 2, 37, cfg.vocab).tolist()
    eng_a = make_engine(cfg, w, max_ctx=128, max_nodes=tree.n_nodes, max_rows=64)
    eng_b = make_engine(cfg, w, max_ctx=128, max_nodes=tree.n_nodes, max_rows=64, keep_logits=False)
    assert eng_a.prefill([prompt]) == eng_b.prefill([prompt])
    for step in range(10):
        if step % 3 == 1:
            cand = [synth.prompt_tokens(step, tree.n_nodes, cfg.vocab, stream=4).tolist()]
            ta, tb = eng_a.step_with_candidates(*args, cand), eng_b.step_with_candidates(*args, cand)
        else:
            ta, tb = eng_a.step(*args), eng_b.step(*args)
        assert ta == tb and eng_a.last_path() == eng_b.last_path() and eng_a.ctx_len() == eng_b.ctx_len()
        da, db = eng_a.drafts(), eng_b.drafts()
        assert da[1] == db[1] and np.array_equal(da[0], db[0])
        with pytest.raises(FirpError) as e:
            eng_b.last_logits()
        assert e.value.code == -2


def test_two_long_sequences_replayed_as_graphs(progress):
    """Two sequences with contexts long enough (and different enough) for the captured-graph
    path: the attention kernel takes each sequence's chunk length from its own committed length
    on the device.  Lockstep with one oracle per sequence; most steps must have been replays."""
    cfg = synth.CONFIGS["tiny_bf16"]
    w = synth.make_weights(cfg, DEV, with_bias=True)
    tree = synth.full_tree((3, 2), "root")
    rep, eng, orcs = run_lockstep_batch(cfg, w, tree, prompt_lens=[640, 531], n_steps=9, tol=2e-2, max_rows=32,
                                        progress=progress)
    assert rep.steps == 9 and sum(rep.accepted_hist[2:]) > 0
    assert eng.stat("graph_launches") >= 7, eng.stat("graph_launches")


def test_default_stream_falls_back_to_direct_launches(progress):
    """The legacy default stream cannot be captured: with graph replay asked for, a context on
    that stream must notice, launch its kernels directly and give the same results as a context
    on a stream of its own."""
    from paper_2410_20488_amd import binding
    cfg = synth.CONFIGS["tiny_bf16"]
    w = synth.make_weights(cfg, DEV, with_bias=True)
    tree = synth.full_tree((3, 2), "root")
    args = (list(tree.parent), list(tree.rank), list(tree.anchor))
    prompt = synth.prompt_tokens(cfg.seed + 9, 600, cfg.vocab).tolist()
    kw = dict(n_layers=cfg.n_layers, d_model=cfg.d_model, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
              head_dim=cfg.head_dim, d_ffn=cfg.d_ffn, vocab=cfg.vocab, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base,
              dtype=cfg.dtype, weights=w, firp_layer=cfg.firp_layer, k=cfg.k, max_ctx=700, max_nodes=tree.n_nodes,
              max_rows=32)
    eng_d = binding.Engine(stream=torch.cuda.default_stream(torch.device(DEV)), **kw)
    eng_s = binding.Engine(**kw)
    for e in (eng_d, eng_s):
        e.set_option("graph", 1)
        e.set_option("keep_logits", 1)
    assert eng_d.prefill([prompt]) == eng_s.prefill([prompt])
    for _ in range(6):
        assert eng_d.step(*args) == eng_s.step(*args)
        assert np.array_equal(eng_d.last_logits(), eng_s.last_logits())
    assert eng_d.stat("graph_launches") == 0 and eng_s.stat("graph_launches") >= 5
