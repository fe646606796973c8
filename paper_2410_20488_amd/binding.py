"""ctypes binding of libfirp.so: the same calls as include/firp.h, argument marshalling only.

PyTorch appears here for device memory (weights, workspace) and the current stream; every
step of the decoding path runs inside the library's kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfirp.so")

FIRP_MAX_K = 8
FIRP_MAX_B = 16
FIRP_MAX_ROWS = 256
STATUS = {0: "FIRP_OK", -1: "FIRP_EINVAL", -2: "FIRP_ESTATE", -3: "FIRP_ECAPACITY", -4: "FIRP_EDEVICE"}


class FirpError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{STATUS.get(code, code)}: {text}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                          "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "max_ctx", "max_batch", "max_nodes", "max_rows", "b_max")]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down",
                                                      "norm_attn", "norm_mlp")] + \
               [("norm_final", C.c_void_p), ("lm_head", C.c_void_p)]


class Tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("parent", C.POINTER(C.c_int32)), ("rank", C.POINTER(C.c_int32)),
                ("anchor", C.POINTER(C.c_uint8))]


_lib = None


def load_library() -> C.CDLL:
    """Load libfirp.so (built by paper_2410_20488_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2410_20488_amd.build` first")
    lib = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    sig = {
        "firp_workspace_bytes": (C.c_size_t, [C.POINTER(ModelDesc), C.c_int32]),
        "firp_init": (C.c_int, [C.POINTER(vp), C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(vp),
                                 C.POINTER(vp), C.c_int32, C.c_int32, vp, C.c_size_t, vp]),
        "firp_init_layers": (C.c_int, [C.POINTER(vp), C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(vp),
                                        C.POINTER(vp), i32p, C.c_int32, vp, C.c_size_t, vp]),
        "firp_build_tree": (C.c_int, [C.POINTER(C.c_float), C.c_int32, C.c_int32, C.c_int32, i32p, i32p, i32p,
                                       C.POINTER(C.c_double)]),
        "firp_train_forward": (C.c_int, [vp, i32p, C.c_int32, C.c_int32, C.POINTER(C.c_double),
                                          C.POINTER(C.c_float)]),
        "firp_prefill": (C.c_int, [vp, C.c_int32, i32p, i32p, i32p]),
        "firp_step": (C.c_int, [vp, C.POINTER(Tree), i32p, i32p]),
        "firp_reset": (C.c_int, [vp]),
        "firp_destroy": (None, [vp]),
        "firp_last_error": (C.c_char_p, [vp]),
        "firp_step_with_candidates": (C.c_int, [vp, C.POINTER(Tree), i32p, i32p, i32p]),
        "firp_check_tree": (C.c_int, [vp, C.POINTER(Tree), i32p]),
        "firp_debug_last_logits": (C.c_int, [vp, C.POINTER(C.c_float), i32p]),
        "firp_debug_last_path": (C.c_int, [vp, i32p]),
        "firp_get_drafts": (C.c_int, [vp, i32p, i32p]),
        "firp_get_ctx_len": (C.c_int, [vp, i32p]),
        "firp_debug_read_cache": (C.c_int, [vp, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float)]),
        "firp_set_option": (C.c_int, [vp, C.c_char_p, C.c_int32]),
        "firp_get_gemm_timing": (C.c_int, [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "firp_get_event_overhead": (C.c_int, [vp, C.POINTER(C.c_double)]),
        "firp_get_stat": (C.c_int, [vp, C.c_char_p, C.POINTER(C.c_int64)]),
        "firp_gemm_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32, C.c_int32]),
        "firp_debug_stream_read": (C.c_int32, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
        "firp_debug_gemm_plan": (C.c_int32, [C.c_int32, C.c_int32, C.c_int32] + [C.POINTER(C.c_int32)] * 5),
        "firp_debug_gemm": (C.c_int, [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp,
                                       C.c_size_t, vp]),
        "firp_gemm_static_capacity": (C.c_size_t, []),
        "firp_debug_gemm_static": (C.c_int, [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTED = ["firp_workspace_bytes", "firp_init", "firp_init_layers", "firp_build_tree", "firp_train_forward", "firp_prefill", "firp_step", "firp_reset", "firp_destroy",
            "firp_last_error", "firp_step_with_candidates", "firp_check_tree", "firp_debug_last_logits", "firp_debug_last_path",
            "firp_get_drafts", "firp_get_ctx_len", "firp_debug_read_cache", "firp_set_option", "firp_get_gemm_timing",
            "firp_gemm_workspace_bytes", "firp_debug_gemm", "firp_debug_gemm_plan", "firp_debug_stream_read",
            "firp_gemm_static_capacity", "firp_debug_gemm_static", "firp_get_event_overhead", "firp_get_stat"]


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p(a: np.ndarray, ty=C.c_int32):
    return a.ctypes.data_as(C.POINTER(ty))


def build_tree(accept, n_nodes: int):
    """Best draft tree of at most `n_nodes` nodes for acceptance rates accept[k][b] (host only).
    Returns (parent, rank, expected tokens per step)."""
    lib = load_library()
    a = np.ascontiguousarray(np.asarray(accept, dtype=np.float32))
    k, b = (a.shape if a.ndim == 2 else (0, 1))
    parent = np.zeros(n_nodes, dtype=np.int32)
    rank = np.zeros(n_nodes, dtype=np.int32)
    n_out = C.c_int32(0)
    expect = C.c_double(0.0)
    rc = lib.firp_build_tree(a.ctypes.data_as(C.POINTER(C.c_float)), k, b, n_nodes, _p(parent), _p(rank),
                             C.byref(n_out), C.byref(expect))
    if rc != 0:
        raise FirpError(rc, "firp_build_tree: invalid argument")
    n = n_out.value
    return parent[:n].tolist(), rank[:n].tolist(), expect.value


def make_tree(parent: Sequence[int], rank: Sequence[int], anchor: Optional[Sequence[int]]):
    """Marshal a topology; returns (Tree struct, keep-alive tuple)."""
    pa, ra = _i32(parent), _i32(rank)
    an = None if anchor is None else np.ascontiguousarray(np.asarray(anchor, dtype=np.uint8))
    t = Tree(len(pa), _p(pa), _p(ra), None if an is None else _p(an, C.c_uint8))
    return t, (pa, ra, an)


def _ptr_array(tensors: Sequence[torch.Tensor]):
    arr = (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    return arr


class Engine:
    """One firp_ctx plus the torch tensors it borrows (weights, workspace)."""

    def __init__(self, *, n_layers: int, d_model: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 d_ffn: int, vocab: int, rms_eps: float, rope_base: float, dtype: str,
                 weights: Dict[str, object], firp_layer: int, k: int, max_ctx: int, max_batch: int = 1,
                 max_nodes: int = 64, max_rows: int = 128, b_max: int = 8,
                 stream: Optional[torch.cuda.Stream] = None, firp_layers: Optional[Sequence[int]] = None):
        self.lib = load_library()
        dev = weights["embed"].device
        if dev.type != "cuda":
            raise ValueError("weights must live on the GPU")
        self.device = dev
        self.k, self.vocab, self.b_max = k, vocab, b_max
        self.desc = ModelDesc(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rms_eps,
                              rope_base, 1 if dtype == "bf16" else 0, max_ctx, max_batch, max_nodes, max_rows,
                              b_max)
        want = torch.bfloat16 if dtype == "bf16" else torch.float32
        self._keep = []
        w = Weights()
        for name in ("embed", "norm_final", "lm_head"):
            t = weights[name]
            assert t.dtype == want and t.is_contiguous() and t.device == dev, name
            setattr(w, name, t.data_ptr())
            self._keep.append(t)
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_mlp"):
            ts = list(weights[name])
            assert len(ts) == n_layers and all(t.dtype == want and t.is_contiguous() for t in ts), name
            arr = _ptr_array(ts)
            setattr(w, name, C.cast(arr, C.POINTER(C.c_void_p)))
            self._keep += [ts, arr]
        pw = pb = None
        if k > 0:
            ts = list(weights["proj_w"])
            assert len(ts) == k and all(t.dtype == want and tuple(t.shape) == (d_model, d_model) for t in ts)
            pw = _ptr_array(ts)
            self._keep += [ts, pw]
            if weights.get("proj_b") is not None:
                tb = list(weights["proj_b"])
                pb = _ptr_array(tb)
                self._keep += [tb, pb]
        nbytes = self.lib.firp_workspace_bytes(C.byref(self.desc), k)
        if nbytes == 0:
            raise FirpError(-1, "invalid model description")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        if os.environ.get("FIRP_POISON_WORKSPACE"):
            # test aid: a workspace of NaN bit patterns shows any read of memory the library has not written
            self.workspace.fill_(0xFF)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        # a stream of its own (default priority): the library replays the step as a captured graph,
        # which the legacy default stream does not allow; everything queued so far (the weights) must
        # be complete before that stream reads it
        self.stream = stream if stream is not None else torch.cuda.Stream(device=dev)
        torch.cuda.synchronize(dev)
        ctx = C.c_void_p()
        pwp = None if pw is None else C.cast(pw, C.POINTER(C.c_void_p))
        pbp = None if pb is None else C.cast(pb, C.POINTER(C.c_void_p))
        if firp_layers is None:
            rc = self.lib.firp_init(C.byref(ctx), C.byref(self.desc), C.byref(w), pwp, pbp, firp_layer, k, base,
                                    nbytes, self.stream.cuda_stream)
        else:      # one prediction layer per step
            assert len(firp_layers) == k
            layers = _i32(list(firp_layers))
            rc = self.lib.firp_init_layers(C.byref(ctx), C.byref(self.desc), C.byref(w), pwp, pbp, _p(layers), k,
                                           base, nbytes, self.stream.cuda_stream)
        if rc != 0:
            raise FirpError(rc, self.lib.firp_last_error(None).decode())
        self.ctx = ctx
        self.batch = 0

    # -- helpers ---------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise FirpError(rc, self.lib.firp_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.firp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the ABI's calls -------------------------------------------------------------------------
    def set_option(self, name: str, value: int):
        self._check(self.lib.firp_set_option(self.ctx, name.encode(), value))

    def prefill(self, prompts: Sequence[Sequence[int]]) -> List[int]:
        lens = _i32([len(p) for p in prompts])
        toks = _i32([t for p in prompts for t in p])
        first = np.zeros(len(prompts), dtype=np.int32)
        self._check(self.lib.firp_prefill(self.ctx, len(prompts), _p(toks), _p(lens), _p(first)))
        self.batch = len(prompts)
        return first.tolist()

    def _run(self, tree, node_tokens=None) -> List[List[int]]:
        t, keep = make_tree(*tree)
        acc = np.zeros((max(self.batch, 1), FIRP_MAX_K + 1), dtype=np.int32)
        n = np.zeros(max(self.batch, 1), dtype=np.int32)
        if node_tokens is None:
            rc = self.lib.firp_step(self.ctx, C.byref(t), _p(acc), _p(n))
        else:
            nt = _i32(node_tokens).reshape(-1)
            rc = self.lib.firp_step_with_candidates(self.ctx, C.byref(t), _p(nt), _p(acc), _p(n))
        self._check(rc)
        del keep
        return [acc[b, :n[b]].tolist() for b in range(self.batch)]

    def step(self, parent, rank, anchor=None) -> List[List[int]]:
        return self._run((parent, rank, anchor))

    def step_with_candidates(self, parent, rank, anchor, node_tokens) -> List[List[int]]:
        return self._run((parent, rank, anchor), node_tokens)

    def reset(self):
        self._check(self.lib.firp_reset(self.ctx))
        self.batch = 0

    def train_forward(self, tokens: Sequence[int], step: int):
        """Training-stage forward for prediction step `step`: (loss, kl[n - step])."""
        t = _i32(list(tokens))
        kl = np.zeros(len(t) - step, dtype=np.float32)
        loss = C.c_double(0.0)
        self._check(self.lib.firp_train_forward(self.ctx, _p(t), len(t), step, C.byref(loss), _p(kl, C.c_float)))
        self.batch = 1
        return loss.value, kl

    def last_logits(self) -> np.ndarray:
        """[batch][T_hi][V] fp32 of the last step."""
        buf = np.empty((self.batch, FIRP_MAX_ROWS, self.vocab), dtype=np.float32)
        n_rows = C.c_int32(0)
        # the library writes rows densely as [batch][T_hi][V]
        self._check(self.lib.firp_debug_last_logits(self.ctx, _p(buf, C.c_float), C.byref(n_rows)))
        t = n_rows.value
        return buf.reshape(-1)[: self.batch * t * self.vocab].reshape(self.batch, t, self.vocab).copy()

    def last_path(self) -> List[List[int]]:
        buf = np.full((self.batch, FIRP_MAX_K + 1), -1, dtype=np.int32)
        self._check(self.lib.firp_debug_last_path(self.ctx, _p(buf)))
        return [[int(v) for v in row if v >= 0] for row in buf]

    def drafts(self):
        d = np.zeros((self.batch, max(self.k, 1), self.b_max), dtype=np.int32)
        valid = np.zeros(self.batch, dtype=np.int32)
        self._check(self.lib.firp_get_drafts(self.ctx, _p(d), _p(valid)))
        return d[:, : self.k], valid.tolist()

    def drafts_valid_host(self) -> List[int]:
        """Whether each sequence has drafts for its next step (the host's mirror: no device work)."""
        valid = np.zeros(self.batch, dtype=np.int32)
        self._check(self.lib.firp_get_drafts(self.ctx, None, _p(valid)))
        return valid.tolist()

    def ctx_len(self) -> List[int]:
        n = np.zeros(self.batch, dtype=np.int32)
        self._check(self.lib.firp_get_ctx_len(self.ctx, _p(n)))
        return n.tolist()

    def gemm_timing(self):
        """(launches, total ms, weight bytes) of the timed projection launches."""
        n, ms, by = C.c_int64(0), C.c_double(0), C.c_double(0)
        self._check(self.lib.firp_get_gemm_timing(self.ctx, C.byref(n), C.byref(ms), C.byref(by)))
        return n.value, ms.value, by.value

    def stat(self, name: str) -> int:
        v = C.c_int64(0)
        self._check(self.lib.firp_get_stat(self.ctx, name.encode(), C.byref(v)))
        return v.value

    def event_bracket_us(self) -> float:
        """Mean reading (microseconds) of an empty pair of events on the library's stream."""
        ms = C.c_double(0)
        self._check(self.lib.firp_get_event_overhead(self.ctx, C.byref(ms)))
        return ms.value * 1e3

    def read_cache(self, seq: int, layer: int):
        n = self.ctx_len()[seq]
        shape = (n, self.desc.n_kv_heads, self.desc.head_dim)
        k = np.zeros(shape, dtype=np.float32)
        v = np.zeros(shape, dtype=np.float32)
        self._check(self.lib.firp_debug_read_cache(self.ctx, seq, layer, _p(k, C.c_float), _p(v, C.c_float)))
        return k, v


def engine_for_config(cfg, weights, *, max_ctx: int, max_batch: int = 1, max_nodes: int = 64, max_rows: int = 128,
                      b_max: int = 8, gemm: Optional[int] = None, keep_logits: bool = False) -> Engine:
    """An Engine for a synthetic model configuration (synth.ModelConfig) and its weight dict.
    `keep_logits`: every step also writes all its logits (read back with Engine.last_logits)."""
    e = Engine(n_layers=cfg.n_layers, d_model=cfg.d_model, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads,
               head_dim=cfg.head_dim, d_ffn=cfg.d_ffn, vocab=cfg.vocab, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base,
               dtype=cfg.dtype, weights=weights, firp_layer=cfg.firp_layer, k=cfg.k, max_ctx=max_ctx,
               max_batch=max_batch, max_nodes=max_nodes, max_rows=max_rows, b_max=b_max, firp_layers=cfg.firp_layers)
    if gemm is not None:
        e.set_option("gemm", gemm)
    if keep_logits:
        e.set_option("keep_logits", 1)
    return e


def debug_gemm(x: torch.Tensor, w: torch.Tensor, kind: int) -> torch.Tensor:
    """y = x . w^T through the library's projection kernel (x fp32 [R,K], w [n,K] fp32 or bf16)."""
    lib = load_library()
    assert x.dtype == torch.float32 and x.is_cuda and x.is_contiguous() and w.is_contiguous()
    rows, kd = x.shape
    n = w.shape[0]
    y = torch.empty(rows, n, dtype=torch.float32, device=x.device)
    nbytes = lib.firp_gemm_workspace_bytes(rows, n, kd)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=x.device)
    if os.environ.get("FIRP_POISON_WORKSPACE"):
        ws.fill_(0xFF)
    base = (ws.data_ptr() + 255) // 256 * 256
    rc = lib.firp_debug_gemm(x.data_ptr(), w.data_ptr(), y.data_ptr(), rows, n, kd,
                             1 if w.dtype == torch.bfloat16 else 0, kind, base, nbytes,
                             torch.cuda.current_stream(x.device).cuda_stream)
    if rc != 0:
        raise FirpError(rc, "firp_debug_gemm")
    return y


def debug_gemm_static(x: torch.Tensor, w: torch.Tensor, y: torch.Tensor) -> None:
    """y = x . w^T through the entry point that allocates nothing (bf16 w; y is the caller's)."""
    lib = load_library()
    assert x.dtype == torch.float32 and y.dtype == torch.float32 and w.dtype == torch.bfloat16
    assert x.is_cuda and x.is_contiguous() and w.is_contiguous() and y.is_contiguous()
    rows, kd = x.shape
    n = w.shape[0]
    assert tuple(y.shape) == (rows, n)
    rc = lib.firp_debug_gemm_static(x.data_ptr(), w.data_ptr(), y.data_ptr(), rows, n, kd,
                                    torch.cuda.current_stream(x.device).cuda_stream)
    if rc != 0:
        raise FirpError(rc, lib.firp_last_error(None).decode())


def gemm_plan(rows: int, n: int, k_dim: int) -> dict:
    """The launch plan the library picks for a projection (host logic only, no GPU needed)."""
    lib = load_library()
    out = [C.c_int32() for _ in range(5)]
    rc = lib.firp_debug_gemm_plan(rows, n, k_dim, *[C.byref(o) for o in out])
    if rc != 0:
        raise FirpError(rc, "firp_debug_gemm_plan")
    return dict(zip(("splits", "k_per_split", "waves", "grid", "row_block"), (o.value for o in out)))


def stream_read_gbps(nbytes: int = 8 << 30, repeats: int = 5, device: str = "cuda:0") -> float:
    """Rate of a plain streaming-read kernel over `nbytes` of device memory (GB/s, best of `repeats`)."""
    lib = load_library()
    buf = torch.zeros(nbytes, dtype=torch.uint8, device=device)
    sink = torch.zeros(1, dtype=torch.int32, device=device)
    stream = torch.cuda.current_stream(buf.device)
    best = 0.0
    for _ in range(repeats + 1):                      # the first pass warms up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        rc = lib.firp_debug_stream_read(buf.data_ptr(), nbytes, sink.data_ptr(), stream.cuda_stream)
        e1.record(stream)
        if rc != 0:
            raise FirpError(rc, "firp_debug_stream_read")
        e1.synchronize()
        best = max(best, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best
