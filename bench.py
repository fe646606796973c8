#!/usr/bin/env python3
"""Benchmark of the FIRP decoding step on one MI355X.

A "step" is one firp_step: the whole hot path (candidate fill, embedding, all decoder layers
with tree attention, the FIRP map, lm-head, greedy verification, draft selection, KV commit)
over one synthetic batch.  Default workload: the LLaMA-2-13B-shaped bf16 model, k = 3, prompt of
1024 uniform-random tokens, the 64-node draft tree, anchors = {root}.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
PROFILES = os.path.join(ROOT, "profiles")


def profile_figures():
    """Figures of the committed rocprofv3 summaries that the bench line quotes: HBM bytes moved
    per weight byte by the projection kernel at the 13B shapes ((FETCH_SIZE + WRITE_SIZE) / weights,
    weighted by each shape's share of a step) and the kernel-trace mean duration of a decode-step
    launch of that kernel.  None where a summary or its line is missing."""
    import re
    out = {"traffic_ratio": None, "trace_avg_launch_us": None}
    for fname, key, pat in (("k_gemm_mfma_13b_shapes_hbm_traffic.md", "traffic_ratio", r"traffic_ratio_13b_step\s*=\s*([0-9.]+)"),
                            ("firp_step_13b_kernel_stats.md", "trace_avg_launch_us", r"decode_launch_trace_mean_us\s*=\s*([0-9.]+)")):
        try:
            with open(os.path.join(PROFILES, fname)) as f:
                m = re.search(pat, f.read())
            if m:
                out[key] = float(m.group(1))
        except OSError:
            pass
    return out


def algorithmic_bytes(cfg, n_nodes: int, t_hi: int, ctx: int, batch: int = 1) -> float:
    """Bytes the method must move in one step: every weight once, and per sequence the live KV
    cache once and the step rows' K/V once out and once in (bf16 = 2 bytes)."""
    e = 2 if cfg.dtype == "bf16" else 4
    kv_row = 2 * cfg.n_kv_heads * cfg.head_dim * e                 # K and V of one row, one layer
    weights = e * (cfg.n_layers * cfg.layer_params() + cfg.vocab * cfg.d_model + cfg.k * cfg.d_model ** 2)
    kv_sweep = ctx * kv_row * cfg.n_layers
    n_anchor = (t_hi - n_nodes) // max(cfg.k, 1)
    step_rows = 2 * kv_row * sum(n_nodes + n_anchor * sum(1 for t in cfg.layers if t <= layer)
                                 for layer in range(cfg.n_layers))
    return float(weights + batch * (kv_sweep + step_rows))


def cpu_baseline(cfg, weights_gpu, tree, prompt, n_steps: int = 3):
    """Time the CPU oracle, as it stands, on the same workload at full depth: its prefill of the
    whole prompt (not timed), then `n_steps` decoding steps with the benchmark's tree."""
    import torch
    from oracle.firp_oracle import FirpOracle

    w = {}
    for k, v in weights_gpu.items():
        w[k] = None if v is None else ([t.cpu() for t in v] if isinstance(v, (list, tuple)) else v.cpu())
    o = FirpOracle(n_layers=cfg.n_layers, d_model=cfg.d_model, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
                   head_dim=cfg.head_dim, d_ffn=cfg.d_ffn, vocab=cfg.vocab, rms_eps=cfg.rms_eps,
                   rope_base=cfg.rope_base, weights=w, firp_layer=cfg.firp_layer, k=cfg.k, b_max=8,
                   dtype=torch.float32, kv_round_bf16=cfg.dtype == "bf16", firp_layers=cfg.firp_layers)
    t_pre = time.perf_counter()
    o.prefill(prompt)
    t0 = time.perf_counter()
    args = dict(parent=list(tree.parent), rank=list(tree.rank), anchor=list(tree.anchor))
    for _ in range(n_steps):
        o.step(**args)
    per_step = (time.perf_counter() - t0) / n_steps
    return {"value": round(per_step * 1e3, 1), "unit": "ms/step", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"fp32 oracle at full depth ({cfg.n_layers} layers): {n_steps} decoding steps of the same tree "
                      f"after its own prefill of the {len(prompt)}-token prompt ({t0 - t_pre:.1f} s, not timed)"}


def accept_pattern_run(eng, cfg, tree, prompts, warmup: int, steps: int):
    """Decode with planted candidates: step i of the rotation carries the true greedy continuation
    for i mod (k+1) levels along the chain of last children (every other candidate is wrong), so
    that many candidates are accepted.  The true continuation comes from plain greedy decoding
    (root-only steps) on the same engine first.  A step whose path ends on a node without pseudo
    rows leaves no drafts: the next call of firp_step then runs the root-only sub-tree by itself
    and counts as a step of its own."""
    import torch
    from paper_2410_20488_amd import synth
    assert len(prompts) == 1, "--accept-pattern runs one sequence"
    prompt, N, k = prompts[0], tree.n_nodes, cfg.k
    targs = (list(tree.parent), list(tree.rank), list(tree.anchor))
    need = (warmup + steps + 2) * (k + 1) + 8
    g = eng.prefill([prompt])
    while len(g) < need:
        g += eng.step([-1], [0], [0])[0]
    emitted = eng.prefill([prompt])
    kids = [[c for c in range(N) if tree.parent[c] == v] for v in range(N)]
    state = {"i": 0, "mismatch": 0, "full": 0, "root_only": 0, "planted": 0}

    def one_step():
        pos = len(emitted)
        valid = eng.drafts_valid_host()[0]
        if not valid:                                     # no drafts: the library runs the root alone
            got = eng.step(*targs)[0]
            state["root_only"] += 1
        else:
            plant = state["i"] % (k + 1)
            state["i"] += 1
            truth = g[pos:pos + k + 1]
            cand = [(t + 7) % cfg.vocab if t in truth else t
                    for t in synth.prompt_tokens(state["i"], N, cfg.vocab, stream=9).tolist()]
            v = 0
            for lvl in range(plant):
                if not kids[v]:
                    break
                v = kids[v][-1]
                cand[v] = g[pos + lvl]
            got = eng.step_with_candidates(*targs, [cand])[0]
            state["full"] += 1
            state["planted"] += plant
        if got != g[pos:pos + len(got)]:
            state["mismatch"] += 1                        # a near-tie between the two launch shapes
        emitted.extend(got)
        return len(got)

    for _ in range(warmup):
        one_step()
    state.update(full=0, root_only=0, planted=0)
    ctx_first = eng.ctx_len()[0]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stamps, tokens = [t0], 0
    for _ in range(steps):
        tokens += one_step()
        stamps.append(time.perf_counter())
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per = sorted((b - a) * 1e3 for a, b in zip(stamps, stamps[1:]))
    return {"ms_per_step": (t1 - t0) * 1e3 / steps, "per_step_ms": per, "tokens": tokens, "ctx_first": ctx_first,
            "full_tree_steps": state["full"], "root_only_steps": state["root_only"],
            "ms_per_token": round((t1 - t0) * 1e3 / max(tokens, 1), 4),
            "continuation_mismatches": state["mismatch"], "topologies_uploaded": eng.stat("topo_uploads")}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="13b", choices=["13b", "7b", "34b", "tiny_bf16", "tiny"],
                    help="13b (default): the headline workload; 7b, 34b: the other LLaMA shapes; tiny: the 4-layer fp32 "
                         "correctness configuration (chain tree, prompt 64); tiny_bf16: the same widths in bf16")
    ap.add_argument("--batch", type=int, default=1, help="independent sequences decoded side by side")
    ap.add_argument("--prompt", type=int, default=0, help="prompt length (default: the configuration's)")
    ap.add_argument("--anchors", default="root", choices=["root", "all"])
    ap.add_argument("--tree", default="", choices=["", "7b", "13b"],
                    help="draft tree of another configuration (13b: the 64-node tree)")
    ap.add_argument("--firp-layers", default="",
                    help="comma-separated prediction layer per step (e.g. 25,30,35: the paper's 13B setting); "
                         "default: the benchmark configuration's single layer")
    ap.add_argument("--accept-pattern", action="store_true",
                    help="instead of the library's own (untrained, never accepted) drafts, plant the true greedy "
                         "continuation so that 0, 1, .. k candidates are accepted in rotation, as trained maps would "
                         "have it: with the root as the only anchor every step that accepts a candidate is followed "
                         "by a root-only step (no drafts)")
    ap.add_argument("--graph", type=int, default=2, choices=[0, 1, 2],
                    help="replay the step as a captured HIP graph: 0 never, 1 whenever possible, 2 (default) the "
                         "library's own rule (only models whose step is short)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy three times (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the step is a single-GPU kernel path); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2410_20488_amd import synth
    from paper_2410_20488_amd import binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": 1 << 30, "copies": 3}))
        return 0
    cfg = synth.CONFIGS[args.config]
    if args.firp_layers:
        import dataclasses
        cfg = dataclasses.replace(cfg, firp_layers=tuple(int(t) for t in args.firp_layers.split(",")))
        assert len(cfg.firp_layers) == cfg.k
    tree = synth.workload_tree(args.tree or args.config, args.anchors)
    prompt_len = args.prompt or {"13b": 1024, "7b": 512, "34b": 2048, "tiny_bf16": 64, "tiny": 64}[args.config]
    t_start = time.time()
    weights = synth.make_weights(cfg, dev)
    torch.cuda.synchronize()
    n_anchor = sum(tree.anchor)
    t_hi = tree.n_nodes + cfg.k * n_anchor
    total_steps = args.warmup + args.steps + 16 + (2 * (args.warmup + args.steps) if args.accept_pattern else 0)
    eng = binding.engine_for_config(cfg, weights, max_ctx=prompt_len + (cfg.k + 1) * (total_steps + 2) + 8,
                      max_batch=args.batch, max_nodes=tree.n_nodes, max_rows=max(128, t_hi), b_max=8)
    eng.set_option("graph", args.graph)
    prompts = [synth.prompt_tokens(cfg.seed, prompt_len, cfg.vocab, stream=b).tolist() for b in range(args.batch)]
    prompt = prompts[0]
    eng.prefill(prompts)
    setup_s = time.time() - t_start
    targs = (list(tree.parent), list(tree.rank), list(tree.anchor))
    pattern = None
    if args.accept_pattern:
        pattern = accept_pattern_run(eng, cfg, tree, prompts, args.warmup, args.steps)
        ms_per_step, per_step, tokens = pattern["ms_per_step"], pattern["per_step_ms"], pattern["tokens"]
        ctx_first, ctx_last = pattern["ctx_first"], eng.ctx_len()[0]
    else:
        for _ in range(args.warmup):
            eng.step(*targs)
        ctx_first = eng.ctx_len()[0]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tokens = 0
        stamps = [t0]   # every step ends with its own host synchronisation (it returns the tokens)
        for _ in range(args.steps):
            tokens += sum(len(t) for t in eng.step(*targs))
            stamps.append(time.perf_counter())
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        per_step = sorted((b - a) * 1e3 for a, b in zip(stamps, stamps[1:]))
        ctx_last = eng.ctx_len()[0]
        ms_per_step = (t1 - t0) * 1e3 / args.steps
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]

    graph_launches = eng.stat("graph_launches")
    # roofline of the dominant kernel (the weight-streaming projection): HIP events on the
    # library's stream around every launch, over 16 further steps
    eng.set_option("time_gemm", 1)
    for _ in range(16):
        eng.step(*targs)
    launches, gemm_ms, gemm_bytes = eng.gemm_timing()
    bracket_us = eng.event_bracket_us()      # what an empty pair of events on the same stream reads
    eng.set_option("time_gemm", 0)
    event_us = gemm_ms * 1e3 / max(launches, 1)
    kernel_us = max(event_us - bracket_us, 1e-3)
    gemm_gbs = gemm_bytes / max(launches, 1) / (kernel_us * 1e-6) / 1e9 if gemm_ms > 0 else 0.0
    prof = profile_figures() if args.config == "13b" and args.anchors == "root" and args.batch == 1 else \
        {"traffic_ratio": None, "trace_avg_launch_us": None}

    # the rate a kernel that only reads can reach on this chip (8 GiB, far beyond every cache)
    ceiling_gbs = binding.stream_read_gbps()

    step_bytes = algorithmic_bytes(cfg, tree.n_nodes, t_hi, (ctx_first + ctx_last) // 2, args.batch)
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "firp_step latency (ms) and achieved HBM GB/s vs peak, 13B-shape bf16, k=3",
        "value": round(ms_per_step, 4), "unit": "ms/step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"LLaMA-2-{args.config.upper()}-shaped decoder, {cfg.dtype} random-init, k={cfg.k} maps at "
                               f"layer {cfg.firp_layer if cfg.firp_layers is None else list(cfg.firp_layers)}, batch {args.batch}, prompt {prompt_len} uniform-random tokens, "
                               f"{tree.n_nodes}-node draft tree, anchors={args.anchors} (T_hi={t_hi}), "
                               f"ctx {ctx_first}->{ctx_last}"},
        "ms_per_step_p10_median_p90": [round(pct(0.1), 4), round(pct(0.5), 4), round(pct(0.9), 4)],
        "step_algorithmic_GB": round(step_bytes / 1e9, 3),
        "step_achieved_GBps": round(step_gbs, 1),
        "step_frac_of_hbm_peak": round(step_gbs / HBM_PEAK_GBS, 4),
        "stream_read_ceiling_GBps": round(ceiling_gbs, 1),
        "step_frac_of_stream_read_ceiling": round(step_gbs / ceiling_gbs, 4),
        "tokens_per_step": round(tokens / args.steps / args.batch, 3),
        "setup_s": round(setup_s, 1),
        "steps_replayed_as_hip_graph": graph_launches,
        "roofline": {"bound": "hbm", "kernel": "k_gemm_mfma", "achieved": round(gemm_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gemm_gbs / HBM_PEAK_GBS, 4),
                     "traffic": (round(prof["traffic_ratio"] * gemm_bytes / max(launches, 1), 0)
                                 if prof["traffic_ratio"] else None),
                     "launches_timed": launches,
                     "avg_launch_us": round(kernel_us, 2),
                     "avg_launch_us_is": "HIP-event bracket around every launch on the library's stream minus the "
                                         "reading of an empty bracket, both measured in this run",
                     "event_bracket_avg_us": round(event_us, 2), "empty_bracket_us": round(bracket_us, 2),
                     "frac_by_raw_event_brackets": round(gemm_bytes / max(gemm_ms, 1e-9) / 1e6 / HBM_PEAK_GBS, 4),
                     "profile_trace_avg_launch_us": prof["trace_avg_launch_us"],
                     "traffic_is": "algorithmic bytes per launch x the (FETCH_SIZE + WRITE_SIZE) / weight-bytes ratio "
                                   "of profiles/k_gemm_mfma_13b_shapes_hbm_traffic.md",
                     "algorithmic_MB_per_launch": round(gemm_bytes / max(launches, 1) / 1e6, 2),
                     "share_of_step_time": round(kernel_us * 1e-3 * launches / 16 / ms_per_step, 3)},
    }
    if pattern is not None:
        out["accept_pattern"] = {k: v for k, v in pattern.items() if k not in ("per_step_ms",)}
    if not args.no_cpu_baseline and args.batch == 1:
        del eng
        out["cpu_baseline"] = cpu_baseline(cfg, weights, tree, prompt)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
