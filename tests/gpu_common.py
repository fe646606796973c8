"""Lock-step comparison of the HIP library (through its C ABI) with the CPU oracle."""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np
import torch

from paper_2410_20488_amd import binding, synth
from tests.helpers import cpu_weights, make_oracle


def make_engine(cfg: synth.ModelConfig, weights, **kw) -> binding.Engine:
    kw.setdefault("keep_logits", True)     # the tests compare all logits of every step
    return binding.engine_for_config(cfg, weights, **kw)


@dataclasses.dataclass
class LockstepReport:
    steps: int = 0
    tokens: int = 0
    max_logit_err: float = 0.0      # max |gpu - oracle| / std(oracle), over all steps
    tie_ambiguous: int = 0          # steps with a near-tie of either kind
    tie_tokens: int = 0             # ... in a committed token (the walk's argmax)
    tie_drafts: int = 0             # ... in the order or the cut of a draft list
    accepted_hist: Optional[List[int]] = None


def logit_error(gpu: np.ndarray, ref: torch.Tensor) -> float:
    ref = ref.to(torch.float64).numpy()
    return float(np.abs(gpu.astype(np.float64) - ref).max() / ref.std())


def _tokens_from_drafts(tree: synth.Tree, depth, drafts, root):
    return [root] + [drafts[depth[v] - 1][tree.rank[v]] for v in range(1, tree.n_nodes)]


def _report_long_layers(orc, progress, min_rows=1024, every=4):
    """A long prompt keeps the oracle busy for minutes: let every few finished layers of such a
    pass write a progress line (a quiet test must be distinguishable from a hung one)."""
    if not progress:
        return
    inner = orc._layer

    def layer(idx, x, *rest, **kw):
        out = inner(idx, x, *rest, **kw)
        if x.shape[0] >= min_rows and (idx + 1) % every == 0:
            progress(f"oracle: layer {idx + 1} of {orc.L} done on {x.shape[0]} rows")
        return out

    orc._layer = layer


def run_lockstep(cfg, weights_gpu, tree: synth.Tree, *, prompt_len: int, n_steps: int, tol: float,
                 gemm=None, b_max=8, with_injection=True, max_rows=128, progress=None, oracle_dtype=torch.float64,
                 max_ctx=None):
    """Prefill both sides with the same prompt, then step both `n_steps` times from the same
    committed state, comparing tokens, path, drafts and all logits after every step (the oracle
    in fp64 unless the caller asks for fp32, which the full-size models do for time).  Every
    third step injects candidates built from the oracle's own greedy continuation so that
    acceptance lengths above one occur with untrained maps.

    Integer results must be identical.  The one exception is a near-tie: when two logits the
    decision compared differ, in the oracle, by no more than the logit tolerance itself (`tol`
    standard deviations of the step's logits: a fixed slack, not one derived from the error the
    kernels happened to make), either order is consistent with the tolerance; such a step is
    counted (committed tokens and draft lists separately) and the GPU side is re-based on the
    oracle's choice (re-prefill with the oracle's committed tokens, or the oracle's candidates
    injected into the next step)."""
    w_cpu = cpu_weights(weights_gpu)
    orc = make_oracle(cfg, w_cpu, dtype=oracle_dtype, b_max=b_max)
    eng = make_engine(cfg, weights_gpu, max_ctx=max_ctx or (prompt_len + (cfg.k + 1) * (n_steps + 2) + 8),
                      max_nodes=max(tree.n_nodes, 1), max_rows=max_rows, b_max=b_max, gemm=gemm)
    prompt = synth.prompt_tokens(cfg.seed, prompt_len, cfg.vocab).tolist()
    rep = LockstepReport(accepted_hist=[0] * (synth.FIRP_MAX_DEPTH + 2))
    _report_long_layers(orc, progress)
    t_o = orc.prefill(prompt)
    t_g = eng.prefill([prompt])[0]
    if progress:
        progress(f"prefill done: oracle {t_o} gpu {t_g}")
    assert t_g == t_o, f"first token differs: gpu {t_g}, oracle {t_o}"
    emitted = [t_o]
    depth = [0] * tree.n_nodes
    for v in range(1, tree.n_nodes):
        depth[v] = depth[tree.parent[v]] + 1
    args = dict(parent=list(tree.parent), rank=list(tree.rank), anchor=list(tree.anchor))
    resync = False          # the GPU's drafts are not the oracle's: drive the next step by injection
    d0, v0 = eng.drafts()
    if orc.drafts is not None and d0[0].tolist() != orc.drafts:
        resync = True
        rep.tie_ambiguous += 1
        rep.tie_drafts += 1
    for step in range(n_steps):
        inject = None
        if with_injection and step % 3 == 2 and max(depth) > 0:
            # candidates along the last-child chain carry the true continuation for 1..k levels
            look = orc.fork()
            look.K, look.V, look.p0 = [t.clone() for t in orc.K], [t.clone() for t in orc.V], orc.p0
            look.root_token, look.drafts = orc.root_token, None
            truth = []
            for _ in range(min(cfg.k, max(depth))):
                truth += look.step(parent=[-1], rank=[0], anchor=[0]).tokens
            inject = synth.prompt_tokens(step, tree.n_nodes, cfg.vocab, stream=5).tolist()
            want_len = 1 + (1 + step // 3) % (len(truth) + 1)
            for v in range(1, tree.n_nodes):
                if inject[v] in truth:
                    inject[v] = (inject[v] + 1) % cfg.vocab
            v = 0
            for lvl in range(want_len - 1):
                kids = [c for c in range(tree.n_nodes) if tree.parent[c] == v]
                if not kids:
                    break
                v = kids[-1]                          # the last sibling: exercises compaction
                inject[v] = truth[lvl]
        elif resync and orc.drafts is not None and tree.n_nodes > 1 and max(depth) <= cfg.k:
            inject = _tokens_from_drafts(tree, depth, orc.drafts, orc.root_token)
        if inject is not None:
            r = orc.step(**args, node_tokens=inject)
            got = eng.step_with_candidates(args["parent"], args["rank"], args["anchor"], [inject])[0]
        elif resync and orc.drafts is None:
            r = orc.step(**args)                     # runs root-only by itself
            got = eng.step_with_candidates([-1], [0], [args["anchor"][0]], [[0]])[0]
        else:
            r = orc.step(**args)
            got = eng.step(args["parent"], args["rank"], args["anchor"])[0]
        resync = False
        lg = eng.last_logits()[0]
        assert lg.shape[0] == r.logits.shape[0], (lg.shape, r.logits.shape)
        ref = r.logits.to(torch.float64).numpy()
        abs_err = float(np.abs(lg.astype(np.float64) - ref).max())
        err = abs_err / float(ref.std())
        rep.max_logit_err = max(rep.max_logit_err, err)
        assert err <= tol, f"step {step}: logit error {err:.3e} > {tol}"
        slack = tol * float(ref.std())
        path_g = eng.last_path()[0]
        if got != r.tokens or path_g != r.path:
            # first position where the two walks part: same node on both sides, other token
            j = next(i for i in range(min(len(got), len(r.tokens)) + 1)
                     if i >= len(got) or i >= len(r.tokens) or got[i] != r.tokens[i])
            assert j < len(got) and j < len(r.tokens) and path_g[:j + 1] == r.path[:j + 1], \
                f"step {step}: walks differ structurally: gpu {got}/{path_g} oracle {r.tokens}/{r.path}"
            row = ref[r.path[j]]
            assert row[got[j]] >= row[r.tokens[j]] - slack, \
                f"step {step}: token {got[j]} vs {r.tokens[j]} differ at margin {row[r.tokens[j]] - row[got[j]]:.3e} > {slack:.3e}"
            rep.tie_ambiguous += 1
            rep.tie_tokens += 1
            emitted += r.tokens
            # re-base on the oracle's committed tokens (its cache holds all but the last of them)
            t = eng.prefill([prompt + emitted[:-1]])[0]
            if t != emitted[-1]:                       # the tie was on the bonus token: both continue from t
                assert j == len(r.tokens) - 1 and t == got[j], f"step {step}: re-based first token {t}"
                emitted[-1] = orc.root_token = t
                orc.drafts = None
            resync = True
        else:
            emitted += r.tokens
            d, valid = eng.drafts()
            assert bool(valid[0]) == (r.drafts is not None), f"step {step}: drafts validity"
            if r.drafts is not None and d[0].tolist() != r.drafts:
                for i in range(cfg.k):
                    row = ref[r.rows.pseudo_row(r.path[-1], i + 1)]
                    g = d[0][i].tolist()
                    assert len(set(g)) == len(g)
                    for a, b in zip(g[:-1], g[1:]):
                        assert row[a] >= row[b] - slack, f"step {step}: draft order beyond tolerance"
                    rest = np.delete(row, g).max()
                    assert row[g[-1]] >= rest - slack, f"step {step}: draft set beyond tolerance"
                rep.tie_ambiguous += 1
                rep.tie_drafts += 1
                resync = True
            assert eng.ctx_len()[0] == orc.p0
        rep.steps += 1
        rep.tokens += len(r.tokens)
        rep.accepted_hist[len(r.tokens)] += 1
        if progress:
            progress(f"step {step}: {len(r.tokens)} tokens, logit err {err:.2e}, ties so far {rep.tie_ambiguous}")
    return rep, eng, orc


def run_lockstep_batch(cfg, weights_gpu, tree: synth.Tree, *, prompt_lens, n_steps: int, tol: float, b_max=8,
                       max_rows=None, progress=None, oracle_dtype=torch.float64):
    """Several sequences decoded side by side by one engine against one oracle per sequence.
    Every step drives both sides with the same candidates, taken from the oracle's state (its
    drafts, or its own greedy continuation planted along the last-child chain on alternating
    steps), so that what the library drafted never feeds forward: its tokens, path, drafts and
    all logits are compared after each step, with the same near-tie rule as `run_lockstep`."""
    B, N, k = len(prompt_lens), tree.n_nodes, cfg.k
    base = make_oracle(cfg, cpu_weights(weights_gpu), dtype=oracle_dtype, b_max=b_max)
    orcs = [base] + [base.fork() for _ in range(B - 1)]
    n_anchor = sum(tree.anchor)
    eng = make_engine(cfg, weights_gpu, max_ctx=max(prompt_lens) + (k + 1) * (n_steps + 2) + 8, max_batch=B,
                      max_nodes=N, max_rows=max_rows or (N + k * n_anchor), b_max=b_max)
    prompts = [synth.prompt_tokens(cfg.seed + 31, n, cfg.vocab, stream=b).tolist() for b, n in enumerate(prompt_lens)]
    first = eng.prefill(prompts)
    for o in orcs:
        _report_long_layers(o, progress)
    assert first == [o.prefill(p) for o, p in zip(orcs, prompts)]
    emitted = [[t] for t in first]
    depth = [0] * N
    for v in range(1, N):
        depth[v] = depth[tree.parent[v]] + 1
    args = dict(parent=list(tree.parent), rank=list(tree.rank), anchor=list(tree.anchor))
    rep = LockstepReport(accepted_hist=[0] * (synth.FIRP_MAX_DEPTH + 2))
    for step in range(n_steps):
        cand = []
        for b, o in enumerate(orcs):
            if (step + b) % 2 == 0 and max(depth) > 0:
                look = o.fork()
                look.K, look.V, look.p0 = [t.clone() for t in o.K], [t.clone() for t in o.V], o.p0
                look.root_token, look.drafts = o.root_token, None
                truth = []
                for _ in range(min(k, max(depth))):
                    truth += look.step(parent=[-1], rank=[0], anchor=[0]).tokens
                t = synth.prompt_tokens(step * 16 + b, N, cfg.vocab, stream=5).tolist()
                t = [(x + 1) % cfg.vocab if x in truth else x for x in t]
                t[0] = o.root_token
                v = 0
                for lvl in range((step // 2 + b) % (len(truth) + 1)):
                    kids = [c for c in range(N) if tree.parent[c] == v]
                    if not kids:
                        break
                    v = kids[-1]
                    t[v] = truth[lvl]
                cand.append(t)
            elif o.drafts is not None:
                cand.append(_tokens_from_drafts(tree, depth, o.drafts, o.root_token))
            else:
                cand.append(None)
        # a sequence without candidates rides along with "no candidate" tokens: both sides then
        # run its root-only step
        res = [o.step(**args, node_tokens=c) if c is not None else o.step(**args) for o, c in zip(orcs, cand)]
        got = eng.step_with_candidates(args["parent"], args["rank"], args["anchor"],
                                       [c if c is not None else [0] + [-1] * (N - 1) for c in cand])
        lg, paths = eng.last_logits(), eng.last_path()
        d, valid = eng.drafts()
        rebase = []
        for b, r in enumerate(res):
            ref = r.logits.to(torch.float64).numpy()
            # the library's rows that the oracle's rows correspond to (a root-only step of the
            # oracle has the root and, if the root is an anchor, its k pseudo rows)
            rows = list(range(ref.shape[0]))
            if r.ran_root_only:
                rows = [0] + ([N + i * n_anchor for i in range(k)] if tree.anchor[0] else [])
            assert len(rows) == ref.shape[0]
            abs_err = float(np.abs(lg[b][rows].astype(np.float64) - ref).max())
            err = abs_err / float(ref.std())
            rep.max_logit_err = max(rep.max_logit_err, err)
            assert err <= tol, f"step {step} sequence {b}: logit error {err:.3e} > {tol}"
            slack = tol * float(ref.std())
            path_g = paths[b] if not r.ran_root_only else r.path
            emitted[b] += r.tokens
            if got[b] != r.tokens or path_g != r.path:
                j = next(i for i in range(min(len(got[b]), len(r.tokens)) + 1)
                         if i >= len(got[b]) or i >= len(r.tokens) or got[b][i] != r.tokens[i])
                assert j < len(got[b]) and j < len(r.tokens) and path_g[:j + 1] == r.path[:j + 1], \
                    f"step {step} sequence {b}: walks differ structurally: {got[b]}/{path_g} vs {r.tokens}/{r.path}"
                row = ref[r.path[j]]
                assert row[got[b][j]] >= row[r.tokens[j]] - slack, f"step {step} sequence {b}: token beyond tolerance"
                rep.tie_ambiguous += 1
                rep.tie_tokens += 1
                rebase.append((b, j == len(r.tokens) - 1, got[b][j]))
                continue
            assert bool(valid[b]) == (r.drafts is not None), f"step {step} sequence {b}: drafts validity"
            if r.drafts is not None and d[b].tolist() != r.drafts:
                for i in range(k):
                    row = ref[r.rows.pseudo_row(r.path[-1], i + 1)]
                    g = d[b][i].tolist()
                    assert len(set(g)) == len(g)
                    for a, c in zip(g[:-1], g[1:]):
                        assert row[a] >= row[c] - slack, f"step {step} sequence {b}: draft order beyond tolerance"
                    assert row[g[-1]] >= np.delete(row, g).max() - slack, f"step {step} sequence {b}: draft set"
                rep.tie_ambiguous += 1
                rep.tie_drafts += 1
            rep.tokens += len(r.tokens)
            rep.accepted_hist[len(r.tokens)] += 1
        if rebase:   # a near-tie changed a committed token: restart every sequence from the oracle's text
            t = eng.prefill([p + e[:-1] for p, e in zip(prompts, emitted)])
            for b, o in enumerate(orcs):
                if t[b] != emitted[b][-1]:             # the tie was on the bonus token: both continue from t
                    assert (b, True, t[b]) in rebase, f"step {step} sequence {b}: re-based first token {t[b]}"
                    emitted[b][-1] = o.root_token = t[b]
                    o.drafts = None
        assert eng.ctx_len() == [o.p0 for o in orcs], f"step {step}: context lengths"
        rep.steps += 1
        if progress:
            progress(f"batch step {step}: {[len(r.tokens) for r in res]} tokens, max logit err "
                     f"{rep.max_logit_err:.2e}, ties so far {rep.tie_ambiguous}")
    return rep, eng, orcs


def compare_cache(eng, orc, cfg, atol=1e-4):
    """Committed K/V of the library against the oracle's.  fp32 caches agree to `atol`; a bf16
    cache holds values both sides rounded to bf16 from slightly different fp32 inputs (the same
    2e-2-of-a-standard-deviation budget as the logits), so an entry may in addition land on the
    neighbouring bf16 value (one unit in the last place, 2^-7 relative at most); the bulk must
    be identical."""
    for layer in range(cfg.n_layers):
        k, v = eng.read_cache(0, layer)
        assert k.shape[0] == orc.p0
        for name, got, ref in (("K", k, orc.K[layer].float().numpy()), ("V", v, orc.V[layer].float().numpy())):
            diff = np.abs(got - ref)
            if cfg.dtype == "f32":
                assert diff.max() <= atol, f"{name} cache layer {layer}"
            else:
                ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
                assert (diff <= 1.001 * ulp + 2e-2 * ref.std()).all(), f"{name} cache layer {layer}: beyond tolerance"
                assert (diff == 0).mean() > 0.5, f"{name} cache layer {layer}: {(diff == 0).mean():.3f} identical"
