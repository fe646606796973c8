"""CPU oracle of the FIRP decoding step.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the HIP library is checked against.  It is
imported by tests/, by the smoke check and by the benchmark's CPU-baseline leg and by
nothing else; the product path never calls it and shares no code with it.

What it computes (paper: Methodology / FIRP, Inference stage, Tree attention; Eq. 1-3):

* a LLaMA-style decoder (the models named in Experiment / Setup): pre-norm RMSNorm, rotary
  position embedding on q and k, softmax attention with grouped KV heads, SwiGLU MLP,
  untied lm-head; every weight is `[out, in]`;
* the FIRP map of Eq. 3, `h~_i = W_i h + b_i` (i = 1..k), applied for every *anchor* node of the
  draft tree to the residual stream that enters decoder layer `t_i`, the prediction layer of
  step i (Training stage: "index of prediction layer for step i"; Setup: three different
  layers for the three steps; `firp_layer` alone means the same layer for every step); pseudo
  hidden state i then runs through the layers from `t_i` on as an extra row with position id
  `pos(anchor) + i` (Training stage: "position id j+i"), seeing the context, the anchor's
  ancestors, the anchor and the earlier pseudo rows of the same anchor (the ablation's "No
  masked" setting; with `t_1 <= t_2 <= ...` an earlier pseudo row always exists already); real
  rows never see pseudo rows (losslessness, Eq. 1);
* tree attention (Tree attention): the flattened tree keeps each node's original position
  `p0 + depth` and a node attends to the cache, its ancestors and itself only;
* greedy verification (Inference stage; greedy sampling in Setup): walk from the root,
  emit the argmax of the current node, descend to the child carrying that token, stop when
  no child does: the accepted path S is the longest one, and `len(S)+1` tokens come out;
* the next draft tree is read off the pseudo rows of the node that ends S: level i gets the
  top-b ids of pseudo row i (ties to the lower id), node v carries `drafts[level-1][rank]`;
* commit: K and V of the accepted path's nodes are appended to the cache;
* the forward pass of the Training stage (Eq. 3-4): the 2n-row sequence of hidden and pseudo
  hidden states with its mask and position ids, and the KL loss (`train_forward`).

Arithmetic is done in `dtype`: fp64 for the pins and the small-model parity tests, fp32 (the
default) where the full-size models would take minutes in fp64.  Weights are whatever bit patterns the caller hands over, widened
exactly.  K and V are optionally rounded to bf16 right after they are produced: that models
a bf16 KV cache as a storage format (the only rounding besides `dtype` itself).

Pins (tests/test_oracle_pins.py): the decoder against the HuggingFace LLaMA implementation
the paper builds on and against torch's library attention / rms_norm; RoPE's relative-
position property; tree attention against brute-force per-path causal runs; pseudo rows
against a brute-force chain with hand-inserted rows; losslessness against cache-free
sequential greedy decoding; forced-acceptance cases; commit == prefill; candidate fill against
a hand-written tree and hand-written draft lists; the next drafts against a plain Python ranking
of the brute-force chain's pseudo-row logits of the node that ends the accepted path (ties
planted); the training forward against per-position causal chains and the library KL routine.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import torch


# --------------------------------------------------------------------------- primitives


def rms_norm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """x / sqrt(mean(x^2) + eps) * gain, row-wise (LLaMA pre-norm)."""
    return x / torch.sqrt((x * x).mean(dim=-1, keepdim=True) + eps) * gain


def rope_rotate(x: torch.Tensor, pos: torch.Tensor, base: float) -> torch.Tensor:
    """Rotary embedding, half-split pairing: dims (j, j + dh/2) rotate by pos * base^(-2j/dh).

    x: [T, H, dh]; pos: [T] integer position ids (the "original positional indices" that
    tree attention preserves)."""
    dh = x.shape[-1]
    half = dh // 2
    # The angle is a function of the integer position alone; it is evaluated in fp64 and only
    # cos/sin are rounded to the working dtype (an fp32 product pos * freq at positions in the
    # thousands would already be off by 1e-4 rad).
    j = torch.arange(half, dtype=torch.float64)
    inv_freq = float(base) ** (-2.0 * j / dh)
    ang = pos.to(torch.float64)[:, None] * inv_freq[None, :]    # [T, half]
    c, s = torch.cos(ang)[:, None, :].to(x.dtype), torch.sin(ang)[:, None, :].to(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


def masked_attention(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                     visible: torch.Tensor) -> torch.Tensor:
    """softmax(q K^T / sqrt(dh)) V over the visible keys of each row.

    q: [T, Hq, dh]; K, V: [S, Hkv, dh]; visible: bool [T, S]; q-head h reads kv-head
    h // (Hq / Hkv).  Returns [T, Hq, dh]."""
    T, Hq, dh = q.shape
    group = Hq // K.shape[1]
    Kq = K.repeat_interleave(group, dim=1)                       # [S, Hq, dh]
    Vq = V.repeat_interleave(group, dim=1)
    scores = torch.einsum("thd,shd->hts", q, Kq) / math.sqrt(dh)
    scores = scores.masked_fill(~visible[None, :, :], float("-inf"))
    p = torch.softmax(scores, dim=-1)
    return torch.einsum("hts,shd->thd", p, Vq)


def round_to_bf16(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.bfloat16).to(x.dtype)


# --------------------------------------------------------------------------- tree parsing


def tree_depths(parent: Sequence[int]) -> List[int]:
    depth = [0] * len(parent)
    for v in range(1, len(parent)):
        assert 0 <= parent[v] < v, "nodes must be in topological order"
        depth[v] = depth[parent[v]] + 1
    return depth


def tree_ancestors(parent: Sequence[int], v: int) -> List[int]:
    """Proper ancestors of v, root first."""
    out = []
    while parent[v] >= 0:
        v = parent[v]
        out.append(v)
    return out[::-1]


@dataclass
class StepRows:
    """Row table of one step: real rows 0..N-1 are the tree nodes, then the pseudo rows, step by
    step: for i = 1..k, the i-th pseudo row of every anchor (ascending node id).  With this order
    the rows that exist at any decoder layer are a prefix of the table."""
    n_nodes: int
    pos_off: List[int]                 # position id minus p0, per row
    sees: List[List[int]]              # step rows visible to each row (including itself)
    pseudo_of: List[tuple]             # per pseudo row: (anchor node, i)
    anchors: List[int]                 # anchor nodes, ascending

    def pseudo_row(self, v: int, i: int) -> int:
        """Row of pseudo hidden state i (1-based) of anchor node v."""
        return self.n_nodes + (i - 1) * len(self.anchors) + self.anchors.index(v)


def build_rows(parent: Sequence[int], anchor: Sequence[int], k: int) -> StepRows:
    n = len(parent)
    depth = tree_depths(parent)
    pos_off = list(depth)
    sees = [tree_ancestors(parent, v) + [v] for v in range(n)]
    anchors = [v for v in range(n) if anchor[v]] if k > 0 else []
    pseudo_of = []
    for i in range(1, k + 1):
        for a, v in enumerate(anchors):
            pos_off.append(depth[v] + i)
            sees.append(sees[v] + [n + (j - 1) * len(anchors) + a for j in range(1, i + 1)])
            pseudo_of.append((v, i))
    return StepRows(n, pos_off, sees, pseudo_of, anchors)


# --------------------------------------------------------------------------- the model


@dataclass
class StepResult:
    tokens: List[int]                  # the a+1 tokens committed by this step, in order
    path: List[int]                    # node ids of the accepted path, root first (a+1 of them)
    logits: torch.Tensor               # [T_hi, V] in the oracle's dtype
    amax: List[int]                    # greedy token of every real row
    node_tokens: List[int]             # token carried by every node of the tree that ran
    rows: StepRows
    drafts: Optional[List[List[int]]]  # next step's candidates [k][b_max], None = invalid
    ran_root_only: bool


class FirpOracle:
    def __init__(self, *, n_layers: int, d_model: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, d_ffn: int, vocab: int, rms_eps: float, rope_base: float,
                 weights: Dict[str, object], firp_layer: int, k: int, b_max: int = 8,
                 dtype: torch.dtype = torch.float32, kv_round_bf16: bool = False,
                 firp_layers: Optional[Sequence[int]] = None):
        self.L, self.d, self.Hq, self.Hkv, self.dh = n_layers, d_model, n_q_heads, n_kv_heads, head_dim
        self.F, self.V, self.eps, self.base = d_ffn, vocab, rms_eps, rope_base
        self.w, self.l, self.k, self.b_max = weights, firp_layer, k, b_max
        self.dtype, self.kv_round = dtype, kv_round_bf16
        # prediction layer t_i of every step i = 1..k (non-decreasing); one value for all by default
        self.layers = [firp_layer] * k if firp_layers is None else [int(t) for t in firp_layers]
        assert len(self.layers) == k and all(0 <= t <= n_layers for t in self.layers)
        assert all(a <= b for a, b in zip(self.layers, self.layers[1:])), "prediction layers must not decrease"
        assert 0 <= firp_layer <= n_layers
        if k > 0:
            # The paper's draft size (0.08 B for 13B, 0.05 B for 7B) is k full d x d maps.
            assert len(weights["proj_w"]) == k
            assert all(tuple(p.shape) == (d_model, d_model) for p in weights["proj_w"])
        self.reset()

    # -- state ----------------------------------------------------------------------
    def reset(self):
        self.K = [torch.zeros(0, self.Hkv, self.dh, dtype=self.dtype) for _ in range(self.L)]
        self.V = [torch.zeros(0, self.Hkv, self.dh, dtype=self.dtype) for _ in range(self.L)]
        self.p0 = 0                      # tokens in the cache
        self.root_token: Optional[int] = None
        self.drafts: Optional[List[List[int]]] = None

    def fork(self) -> "FirpOracle":
        """A fresh sequence sharing the same weights."""
        o = object.__new__(FirpOracle)
        o.__dict__.update(self.__dict__)
        o.reset()
        return o

    def _W(self, name: str, layer: Optional[int] = None) -> torch.Tensor:
        t = self.w[name] if layer is None else self.w[name][layer]
        return t.to(self.dtype)

    # -- one decoder layer on a set of rows ---------------------------------------------
    def _layer(self, layer: int, x: torch.Tensor, pos: torch.Tensor, K_ctx: torch.Tensor,
               V_ctx: torch.Tensor, visible: torch.Tensor):
        """x: [T, d] residual stream of the rows; K_ctx/V_ctx: [S_ctx, Hkv, dh] cache of this
        layer; visible: bool [T, S_ctx + T] over (cache slots, then the rows themselves).
        Returns (new x, K of the rows, V of the rows)."""
        T = x.shape[0]
        a = rms_norm(x, self._W("norm_attn", layer), self.eps)
        q = (a @ self._W("wq", layer).T).view(T, self.Hq, self.dh)
        kk = (a @ self._W("wk", layer).T).view(T, self.Hkv, self.dh)
        vv = (a @ self._W("wv", layer).T).view(T, self.Hkv, self.dh)
        q = rope_rotate(q, pos, self.base)
        kk = rope_rotate(kk, pos, self.base)
        if self.kv_round:
            kk, vv = round_to_bf16(kk), round_to_bf16(vv)
        o = masked_attention(q, torch.cat([K_ctx, kk]), torch.cat([V_ctx, vv]), visible)
        x = x + o.reshape(T, self.Hq * self.dh) @ self._W("wo", layer).T
        b = rms_norm(x, self._W("norm_mlp", layer), self.eps)
        g = b @ self._W("w_gate", layer).T
        u = b @ self._W("w_up", layer).T
        x = x + (torch.nn.functional.silu(g) * u) @ self._W("w_down", layer).T
        return x, kk, vv

    def _logits(self, x: torch.Tensor) -> torch.Tensor:
        return rms_norm(x, self._W("norm_final"), self.eps) @ self._W("lm_head").T

    def _embed(self, tokens: Sequence[int]) -> torch.Tensor:
        idx = torch.as_tensor(list(tokens), dtype=torch.long)
        return self.w["embed"][idx].to(self.dtype)

    # -- plain causal forward (the textbook definition; used by greedy and by prefill) ------
    def causal_forward(self, tokens: Sequence[int], keep_cache: bool = False) -> torch.Tensor:
        """Logits [n, V] of a plain causal pass over `tokens` starting from an empty context."""
        n = len(tokens)
        x = self._embed(tokens)
        pos = torch.arange(n)
        visible = torch.tril(torch.ones(n, n, dtype=torch.bool))
        empty = torch.zeros(0, self.Hkv, self.dh, dtype=self.dtype)
        Ks, Vs = [], []
        for layer in range(self.L):
            x, kk, vv = self._layer(layer, x, pos, empty, empty, visible)
            Ks.append(kk)
            Vs.append(vv)
        if keep_cache:
            self.K, self.V, self.p0 = Ks, Vs, n
        return self._logits(x)

    def greedy(self, prompt: Sequence[int], m: int) -> List[int]:
        """Sequential greedy decoding with NO cache: every token from a full causal pass.
        This is P of Eq. 1: what any lossless scheme must reproduce."""
        seq = list(prompt)
        out = []
        for _ in range(m):
            t = int(torch.argmax(self.causal_forward(seq)[-1]))   # first max = lowest id
            out.append(t)
            seq.append(t)
        return out

    # -- Training stage, forward only ---------------------------------------------------------
    def train_forward(self, tokens: Sequence[int], step: int):
        """Forward pass of the Training stage for prediction step `step` (1-based) on one
        sequence X_1..X_n, from an empty context; the KL loss of Eq. 4 and its terms.

        The n hidden states entering layer t_step are mapped (Eq. 3) to n pseudo hidden states
        and appended: rows [h_1..h_n, h~_1..h~_n].  h~_j stands for position j + step: it sees
        h_1 .. h_{j+step-1} and itself (the rows that exist: at most h_n) and carries position
        id j + step; the real rows stay causal among themselves.  All 2n rows pass the
        remaining layers and the lm-head; loss = sum_{q=1}^{n-step} KL(P~_q, P_{q+step}), with
        KL(A, B) = sum_t A_t (log A_t - log B_t).
        Returns (loss, kl[n - step], logits[2n, V])."""
        n, i = len(tokens), int(step)
        assert 1 <= i <= self.k and n > i
        t_i = self.layers[i - 1]
        empty = torch.zeros(0, self.Hkv, self.dh, dtype=self.dtype)
        x = self._embed(tokens)
        causal = torch.tril(torch.ones(n, n, dtype=torch.bool))
        for layer in range(t_i):
            x, _, _ = self._layer(layer, x, torch.arange(n), empty, empty, causal)
        pseudo = x @ self._W("proj_w", i - 1).T
        if self.w.get("proj_b") is not None:
            pseudo = pseudo + self._W("proj_b", i - 1)
        x = torch.cat([x, pseudo])
        pos = torch.cat([torch.arange(n), torch.arange(n) + i])      # 0-based position ids
        vis = torch.zeros(2 * n, 2 * n, dtype=torch.bool)
        vis[:n, :n] = causal
        for j in range(n):                                           # 0-based j: pseudo row of h_{j+1}
            vis[n + j, : min(j + i, n)] = True                       # h_1 .. h_{j+1+step-1}
            vis[n + j, n + j] = True
        for layer in range(t_i, self.L):
            x, _, _ = self._layer(layer, x, pos, empty, empty, vis)
        logits = self._logits(x)
        logp = torch.log_softmax(logits, dim=-1)
        kl = torch.stack([(logp[n + q].exp() * (logp[n + q] - logp[q + i])).sum() for q in range(n - i)])
        return float(kl.sum()), kl, logits

    # -- the FIRP step ---------------------------------------------------------------------
    def prefill(self, tokens: Sequence[int]) -> int:
        """Fill the cache with tokens[:-1], then run a root-only step on tokens[-1] so that
        the first generated token and the first drafts exist.  Returns that token."""
        assert len(tokens) >= 1
        self.reset()
        if len(tokens) > 1:
            self.causal_forward(tokens[:-1], keep_cache=True)
        self.root_token = int(tokens[-1])
        self.drafts = None
        res = self.step(parent=[-1], rank=[0], anchor=[1])
        return res.tokens[0]

    def step(self, parent: Sequence[int], rank: Sequence[int], anchor: Optional[Sequence[int]] = None,
             node_tokens: Optional[Sequence[int]] = None) -> StepResult:
        assert self.root_token is not None, "step before prefill"
        n_full = len(parent)
        anchor = [1] * n_full if anchor is None else list(anchor)
        parent, rank = list(parent), list(rank)
        root_only = False
        if node_tokens is not None:                      # injected candidates (tests)
            tok = [self.root_token] + [int(t) for t in node_tokens[1:]]
        elif self.drafts is not None and n_full > 1:
            depth = tree_depths(parent)
            assert max(depth) <= self.k, "tree deeper than the number of pseudo states"
            tok = [self.root_token] + [self.drafts[depth[v] - 1][rank[v]] for v in range(1, n_full)]
        else:                                            # no drafts: the root-only sub-tree
            root_only = n_full > 1
            parent, rank, anchor = [-1], [0], [anchor[0]]
            tok = [self.root_token]

        rows = build_rows(parent, anchor, self.k)
        N, T_hi, p0 = rows.n_nodes, len(rows.pos_off), self.p0
        pos = p0 + torch.as_tensor(rows.pos_off)

        def visible_for(n_rows: int) -> torch.Tensor:
            vis = torch.zeros(n_rows, p0 + n_rows, dtype=torch.bool)
            vis[:, :p0] = True
            for r in range(n_rows):
                vis[r, [p0 + c for c in rows.sees[r]]] = True
            return vis

        # Rows present at decoder layer `layer`: the nodes and every pseudo row whose prediction
        # layer is <= layer.  Eq. 3 is applied to the residual stream entering layer t_i.
        nA = len(rows.anchors)

        def add_pseudo(x: torch.Tensor, i: int) -> torch.Tensor:
            new_rows = []
            for v in rows.anchors:
                h = self._W("proj_w", i - 1) @ x[v]
                if self.w.get("proj_b") is not None:
                    h = h + self._W("proj_b", i - 1)
                new_rows.append(h)
            return torch.cat([x, torch.stack(new_rows)], dim=0)

        x = self._embed(tok)
        step_K: List[torch.Tensor] = []
        step_V: List[torch.Tensor] = []
        vis_cache: Dict[int, torch.Tensor] = {}
        for layer in range(self.L + 1):
            if nA:
                for i in range(1, self.k + 1):
                    if self.layers[i - 1] == layer:
                        x = add_pseudo(x, i)
            if layer == self.L:
                break
            n_rows = x.shape[0]
            if n_rows not in vis_cache:
                vis_cache[n_rows] = visible_for(n_rows)
            x, kk, vv = self._layer(layer, x, pos[:n_rows], self.K[layer], self.V[layer], vis_cache[n_rows])
            step_K.append(kk)
            step_V.append(vv)
        assert x.shape[0] == T_hi

        logits = self._logits(x)
        amax = [int(torch.argmax(logits[r])) for r in range(N)]

        # greedy verification: longest accepted path
        children: List[List[int]] = [[] for _ in range(N)]
        for v in range(1, N):
            children[parent[v]].append(v)
        cur, path, out = 0, [0], []
        while True:
            t = amax[cur]
            out.append(t)
            nxt = next((c for c in children[cur] if tok[c] == t), None)
            if nxt is None:
                break
            cur = nxt
            path.append(cur)
        assert 1 <= len(out) <= max(tree_depths(parent)) + 1

        # next drafts from the pseudo rows of the node that ends the path
        drafts = None
        if anchor[cur] and self.k > 0:
            drafts = []
            for i in range(1, self.k + 1):
                # stable descending sort: equal logits keep ascending id order
                order = torch.sort(logits[rows.pseudo_row(cur, i)], descending=True, stable=True).indices.tolist()
                drafts.append([int(t_) for t_ in order[: self.b_max]])

        # commit the accepted path
        sel = torch.as_tensor(path)
        for layer in range(self.L):
            self.K[layer] = torch.cat([self.K[layer], step_K[layer][sel]])
            self.V[layer] = torch.cat([self.V[layer], step_V[layer][sel]])
        self.p0 += len(path)
        self.root_token = out[-1]
        self.drafts = drafts
        return StepResult(out, path, logits, amax, tok, rows, drafts, root_only)
