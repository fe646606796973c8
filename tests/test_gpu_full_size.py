"""Parity at the benchmark's full sizes: the LLaMA-2-7B- and 13B-shaped models at full depth,
their prompts and draft trees, in the launch configuration bench.py times, against the CPU
oracle run on the same weights (all logits of every step, tokens, path, drafts)."""
import pytest
import torch

from paper_2410_20488_amd import synth
from tests.gpu_common import run_lockstep

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,prompt_len,n_steps,layers", [("7b", 512, 4, None), ("13b", 1024, 3, None),
                                                            ("7b", 256, 3, (15, 20, 25))])
def test_full_depth_model_matches_oracle(name, prompt_len, n_steps, layers, progress):
    """`layers`: one prediction layer per step (15/20/25 is the paper's setting for the 7B models)."""
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[name]
    if layers is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, firp_layers=layers)
    progress(f"{name}: generating weights")
    w = synth.make_weights(cfg, dev)
    tree = synth.workload_tree(name)
    rep, eng, orc = run_lockstep(cfg, w, tree, prompt_len=prompt_len, n_steps=n_steps, tol=2e-2,
                                 progress=progress, max_rows=128)
    progress(f"{name}: max logit err {rep.max_logit_err:.3e}, ties {rep.tie_ambiguous}, "
             f"accepted histogram {rep.accepted_hist}")
    assert rep.steps == n_steps
    assert rep.tie_ambiguous <= n_steps        # near-ties are rare, not the rule


def test_34b_widths_batch_of_four(progress):
    """The launch configuration of the 34B-shaped workload (grouped-query attention with 64 query
    and 8 key/value heads, width 8192, FFN 22016, four sequences x 67 rows = 268 rows in every
    projection) at a depth the oracle finishes in seconds: 4 of the 48 layers, the maps at layer 2."""
    from tests.gpu_common import run_lockstep_batch
    dev = torch.device("cuda:0")
    cfg = synth.scaled_config(synth.CONFIGS["34b"], 4, 2)
    progress("34b widths: generating weights")
    w = synth.make_weights(cfg, dev)
    tree = synth.workload_tree("34b")
    rep, eng, orcs = run_lockstep_batch(cfg, w, tree, prompt_lens=[96, 17, 64, 130], n_steps=4, tol=2e-2,
                                        progress=progress)
    progress(f"34b widths: max logit err {rep.max_logit_err:.3e}, ties {rep.tie_ambiguous}, "
             f"accepted histogram {rep.accepted_hist}")
    assert rep.steps == 4
    assert rep.tie_ambiguous <= 8               # of 16 (sequence, step) pairs
    assert sum(rep.accepted_hist[2:]) > 0        # planted continuations were accepted
