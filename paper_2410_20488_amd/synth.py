"""Seeded synthetic inputs: model shapes, weights, prompts and draft-tree topologies.

This module serves both the HIP path and the CPU oracle and therefore holds none of the
method's arithmetic: it only *produces inputs* (random-init weights, uniform-random
prompts, static tree topologies given as parent/rank arrays).  What a tree means (masks,
depths, position ids, the verify walk) is implemented separately on each side.

Stand-in for the paper's workloads (Experiment / Setup and Datasets): the paper decodes
XSum, GSM8K and MT-bench prompts with LLaMA-2-Chat / Vicuna 7B and 13B weights and
ShareGPT-trained maps.  Neither datasets nor weights are available, and the measured
quantity (cost of one decoding step) depends on shapes only, so prompts are uniform-random
token ids and every weight is N(0, 0.02) from a counter-based generator.

The generator is integer-only up to one final fp32 multiply, so any element can be
regenerated bit-identically on the CPU and on the GPU:
    u64    = splitmix64(seed ^ (tensor_id << 40) ^ (3*index + j)),  j = 0, 1, 2
    normal = scale * (sum of the twelve 16-bit fields of the three hashes / 65536 - 6)
(an Irwin-Hall approximation of a unit normal), then rounded to the model dtype.
"""
from __future__ import annotations

import dataclasses
import itertools
from typing import Dict, List, Optional, Tuple

import torch

_MASK64 = (1 << 64) - 1


def _i64(v: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _splitmix64(z: torch.Tensor) -> torch.Tensor:
    z = z + _i64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _i64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _i64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


def splitmix64_py(z: int) -> int:
    """Pure-Python reference of the same hash (used by the generator's own test)."""
    z = (z + 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def normal_tensor(seed: int, tensor_id: int, shape: Tuple[int, ...], scale: float,
                  dtype: torch.dtype, device: str | torch.device = "cpu",
                  offset: float = 0.0, chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of `offset + scale * approx-N(0,1)`, identical on every device."""
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(n, dtype=dtype, device=device)
    base = _i64(seed ^ (tensor_id << 40))
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device) * 3
        acc = torch.zeros(hi - lo, dtype=torch.int64, device=device)
        for j in range(3):
            h = _splitmix64((idx + j) ^ base)
            for f in range(4):
                acc += _lsr(h, 16 * f) & 0xFFFF
        val = (acc - 6 * 65536).to(torch.float32) * (scale / 65536.0)
        if offset != 0.0:
            val = val + offset
        out[lo:hi] = val.to(dtype)
    return out.view(*shape)


def prompt_tokens(seed: int, length: int, vocab: int, stream: int = 0) -> torch.Tensor:
    """Uniform-random token ids (int32, CPU): splitmix64(seed ^ tag ^ j) mod vocab."""
    j = torch.arange(length, dtype=torch.int64)
    h = _splitmix64(j ^ _i64(seed ^ (0xF1 << 48) ^ (stream << 32)))
    return (_lsr(h, 1) % vocab).to(torch.int32)


# ----------------------------------------------------------------------------- shapes


@dataclasses.dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    firp_layer: int            # pseudo rows are inputs to this 0-based decoder layer
    k: int                     # number of pseudo hidden states per anchor
    dtype: str = "bf16"        # "bf16" or "f32": weights and KV cache
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    seed: int = 20488
    firp_layers: Optional[Tuple[int, ...]] = None   # prediction layer of every step; None = firp_layer for all

    @property
    def layers(self) -> Tuple[int, ...]:
        return tuple(self.firp_layers) if self.firp_layers is not None else (self.firp_layer,) * self.k

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    def layer_params(self) -> int:
        d, hq, hkv, dh, f = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn
        return d * hq * dh * 2 + d * hkv * dh * 2 + 3 * d * f

    def weight_bytes(self) -> int:
        e = 2 if self.dtype == "bf16" else 4
        return e * (self.n_layers * self.layer_params() + self.vocab * self.d_model
                    + self.k * self.d_model * self.d_model)


# The five workload shapes (index = position in the benchmark's config list).
CONFIGS: Dict[str, ModelConfig] = {
    "tiny": ModelConfig("tiny", 4, 256, 4, 4, 64, 688, 1024, firp_layer=2, k=3, dtype="f32",
                        rms_eps=1e-6, seed=20488),
    "tiny_bf16": ModelConfig("tiny_bf16", 4, 256, 4, 4, 64, 688, 1024, firp_layer=2, k=3,
                             dtype="bf16", rms_eps=1e-6, seed=20488),
    "tiny_gqa": ModelConfig("tiny_gqa", 3, 256, 8, 2, 32, 352, 520, firp_layer=1, k=2,
                            dtype="bf16", rms_eps=1e-5, seed=20493),
    "7b": ModelConfig("7b", 32, 4096, 32, 32, 128, 11008, 32000, firp_layer=16, k=3, seed=20489),
    "13b": ModelConfig("13b", 40, 5120, 40, 40, 128, 13824, 32000, firp_layer=20, k=3, seed=20490),
    "34b": ModelConfig("34b", 48, 8192, 64, 8, 128, 22016, 32000, firp_layer=24, k=3, seed=20492),
}


def scaled_config(base: ModelConfig, n_layers: int, firp_layer: int, name: Optional[str] = None,
                  **kw) -> ModelConfig:
    """Same widths as `base`, fewer layers: a parity case the oracle finishes quickly."""
    kw.setdefault("firp_layers", None)   # per-step layers of the full model do not carry over
    return dataclasses.replace(base, name=name or f"{base.name}_L{n_layers}", n_layers=n_layers,
                               firp_layer=firp_layer, **kw)


# tensor ids of the generator (fixed enumeration)
_T_EMBED, _T_LM, _T_NF = 1, 2, 3
_T_LAYER0, _T_PER_LAYER = 16, 16
_L_WQ, _L_WK, _L_WV, _L_WO, _L_WG, _L_WU, _L_WD, _L_N1, _L_N2 = range(9)
_T_PROJ_W, _T_PROJ_B = 4096, 4160


def make_weights(cfg: ModelConfig, device: str | torch.device = "cpu", with_bias: bool = False,
                 std: float = 0.02) -> Dict[str, object]:
    """Random-init weights of `cfg` on `device`, all `[out, in]` row-major in the model dtype.

    Norm gains are 1 + 0.1*N(0,1) (so that a mis-indexed gain is visible); FIRP maps are k
    full d x d matrices (the paper's draft sizes 0.08 B / 0.05 B equal 3*d^2) and optional
    biases of length d.
    """
    dt, sd = cfg.torch_dtype, cfg.seed
    d, hq, hkv, dh, f, v = cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab

    def nrm(tid, shape, scale=std, offset=0.0):
        return normal_tensor(sd, tid, shape, scale, dt, device, offset)

    w: Dict[str, object] = {
        "embed": nrm(_T_EMBED, (v, d)),
        "lm_head": nrm(_T_LM, (v, d)),
        "norm_final": nrm(_T_NF, (d,), 0.1, 1.0),
    }
    names = ["wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp"]
    shapes = [(hq * dh, d), (hkv * dh, d), (hkv * dh, d), (d, hq * dh), (f, d), (f, d), (d, f), (d,), (d,)]
    for nm in names:
        w[nm] = []
    for layer in range(cfg.n_layers):
        for j, (nm, shp) in enumerate(zip(names, shapes)):
            tid = _T_LAYER0 + layer * _T_PER_LAYER + j
            if nm.startswith("norm"):
                w[nm].append(nrm(tid, shp, 0.1, 1.0))
            else:
                w[nm].append(nrm(tid, shp))
    w["proj_w"] = [nrm(_T_PROJ_W + i, (d, d)) for i in range(cfg.k)]
    w["proj_b"] = [nrm(_T_PROJ_B + i, (d,)) for i in range(cfg.k)] if with_bias else None
    return w


# ----------------------------------------------------------------------------- trees


@dataclasses.dataclass(frozen=True)
class Tree:
    """Static draft-tree topology: node 0 is the root (the last committed token), nodes are
    in topological (BFS) order, `rank[v]` says which of the top-b candidates of its level
    node v carries, `anchor[v]` marks the nodes whose hidden state is projected to k pseudo
    hidden states."""
    parent: Tuple[int, ...]
    rank: Tuple[int, ...]
    anchor: Tuple[int, ...]

    @property
    def n_nodes(self) -> int:
        return len(self.parent)


def _tree_from_paths(paths: List[Tuple[int, ...]], anchors: str) -> Tree:
    paths = sorted(paths, key=lambda p: (len(p), p))
    assert paths[0] == ()
    index = {p: i for i, p in enumerate(paths)}
    parent = tuple(-1 if not p else index[p[:-1]] for p in paths)
    rank = tuple(0 if not p else p[-1] for p in paths)
    if anchors == "root":
        anchor = tuple(1 if i == 0 else 0 for i in range(len(paths)))
    elif anchors == "all":
        anchor = tuple(1 for _ in paths)
    elif anchors == "none":
        anchor = tuple(0 for _ in paths)
    else:
        raise ValueError(anchors)
    return Tree(parent, rank, anchor)


def chain_tree(depth: int, anchors: str = "root") -> Tree:
    """Root plus one candidate per future position (rank 0 at every level)."""
    return _tree_from_paths([tuple([0] * j) for j in range(depth + 1)], anchors)


def full_tree(branching: Tuple[int, ...], anchors: str = "root") -> Tree:
    """Complete tree with top-b_i branching at level i (4/3/2 gives 1 + 40 nodes)."""
    paths: List[Tuple[int, ...]] = [()]
    for depth in range(1, len(branching) + 1):
        paths += list(itertools.product(*[range(b) for b in branching[:depth]]))
    return _tree_from_paths(paths, anchors)


def budget_tree(branching: Tuple[int, ...], n_candidates: int, anchors: str = "root") -> Tree:
    """Root plus the `n_candidates` nodes of the full `branching` tree with the smallest
    product of (rank+1) along their path, ties by (depth, lexicographic).  Ancestor-closed.
    Stands in for the searched 63-node tree of the paper's experiments (8/4/2, 63 -> 64 nodes)."""
    cand: List[Tuple[int, ...]] = []
    for depth in range(1, len(branching) + 1):
        cand += list(itertools.product(*[range(b) for b in branching[:depth]]))

    def cost(p):
        c = 1
        for r in p:
            c *= r + 1
        return c

    cand.sort(key=lambda p: (cost(p), len(p), p))
    chosen = cand[:n_candidates]
    chosen_set = set(chosen)
    for p in chosen:                      # ancestor-closed by monotonicity of the cost
        assert not p[:-1] or p[:-1] in chosen_set
    return _tree_from_paths([()] + chosen, anchors)


def random_tree(seed: int, n_nodes: int, max_depth: int, max_rank: int, anchor_prob: float) -> Tree:
    """Irregular topology for edge-case tests: random parents, distinct ranks per sibling set."""
    g = torch.Generator().manual_seed(seed)
    paths: List[Tuple[int, ...]] = [()]
    tries = 0
    while len(paths) < n_nodes and tries < 10000:
        tries += 1
        p = paths[int(torch.randint(len(paths), (1,), generator=g))]
        if len(p) >= max_depth:
            continue
        q = p + (int(torch.randint(max_rank, (1,), generator=g)),)
        if q not in paths:
            paths.append(q)
    t = _tree_from_paths(paths, "none")
    anchor = tuple(int(torch.rand((), generator=g) < anchor_prob) for _ in t.parent)
    return Tree(t.parent, t.rank, anchor)


def with_anchors(tree: Tree, anchors: str) -> Tree:
    n = tree.n_nodes
    a = {"root": [1] + [0] * (n - 1), "all": [1] * n, "none": [0] * n}[anchors]
    return Tree(tree.parent, tree.rank, tuple(a))


def workload_tree(config_name: str, anchors: str = "root") -> Tree:
    """The tree each benchmark configuration uses."""
    if config_name.startswith("tiny"):
        return chain_tree(3 if config_name != "tiny_gqa" else 2, anchors)
    if config_name == "7b":
        return full_tree((4, 3, 2), anchors)
    return budget_tree((8, 4, 2), 63, anchors)

FIRP_MAX_DEPTH = 8   # deepest tree level the library accepts
