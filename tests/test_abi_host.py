"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and
its host-side validation (done before anything is enqueued) returns the documented codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2410_20488_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2410_20488_amd import build
        build.build(verbose=False)
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "firp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(firp_[a-z_]+)\s*\(", header)))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in firp.h but not exported"
    assert sorted(binding.EXPORTED) == declared


def _desc(**kw):
    base = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=128,
                rms_eps=1e-5, rope_base=10000.0, dtype=1, max_ctx=64, max_batch=2, max_nodes=8, max_rows=16,
                b_max=4)
    base.update(kw)
    return binding.ModelDesc(*[base[n] for n, _ in binding.ModelDesc._fields_])


def test_workspace_bytes_and_bad_descriptions(lib):
    good = _desc()
    n = lib.firp_workspace_bytes(C.byref(good), 2)
    assert n > 0 and n % 256 == 0
    assert lib.firp_workspace_bytes(C.byref(_desc(max_ctx=128)), 2) > n
    for bad in (dict(n_q_heads=3), dict(head_dim=15), dict(dtype=7), dict(max_rows=4), dict(max_rows=300),
                dict(b_max=0), dict(b_max=17), dict(vocab=1), dict(rms_eps=0.0)):
        assert lib.firp_workspace_bytes(C.byref(_desc(**bad)), 2) == 0, bad
    assert lib.firp_workspace_bytes(C.byref(good), 9) == 0
    assert lib.firp_workspace_bytes(None, 1) == 0


class _HostCtx:
    """A context over fake (never dereferenced) device pointers: init only records them."""

    def __init__(self, lib, k=2, **kw):
        self.lib = lib
        self.desc = _desc(**kw)
        L = self.desc.n_layers
        fake = 0x10000
        self.arr = (C.c_void_p * L)(*([fake] * L))
        w = binding.Weights()
        for name, _ in binding.Weights._fields_:
            if name in ("embed", "norm_final", "lm_head"):
                setattr(w, name, fake)
            else:
                setattr(w, name, C.cast(self.arr, C.POINTER(C.c_void_p)))
        self.w = w
        self.pw = (C.c_void_p * max(k, 1))(*([fake] * max(k, 1)))
        self.k = k
        self.ctx = C.c_void_p()

    def init(self, layer=1, workspace=0x100000, nbytes=None, weights=True, proj=True):
        if nbytes is None:
            nbytes = self.lib.firp_workspace_bytes(C.byref(self.desc), self.k)
        return self.lib.firp_init(C.byref(self.ctx), C.byref(self.desc), C.byref(self.w) if weights else None,
                                  C.cast(self.pw, C.POINTER(C.c_void_p)) if proj else None, None, layer, self.k,
                                  workspace, nbytes, None)

    def close(self):
        if self.ctx:
            self.lib.firp_destroy(self.ctx)
            self.ctx = C.c_void_p()


def test_init_argument_errors(lib):
    h = _HostCtx(lib)
    assert h.init(layer=3) == -1 and b"layer_l" in lib.firp_last_error(None)
    assert h.init(weights=False) == -1
    assert h.init(proj=False) == -1
    assert h.init(workspace=0) == -1
    assert h.init(workspace=0x100010) == -1 and b"aligned" in lib.firp_last_error(None)
    assert h.init(nbytes=1024) == -3
    assert not h.ctx
    assert h.init() == 0 and h.ctx
    h.close()


def test_init_layers_argument_errors(lib):
    """One prediction layer per step: entries inside [0, n_layers] and not decreasing."""
    h = _HostCtx(lib, k=3)
    nbytes = lib.firp_workspace_bytes(C.byref(h.desc), 3)
    L = h.desc.n_layers

    def init(layers):
        arr = (C.c_int32 * 3)(*layers) if layers is not None else None
        return lib.firp_init_layers(C.byref(h.ctx), C.byref(h.desc), C.byref(h.w),
                                    C.cast(h.pw, C.POINTER(C.c_void_p)), None, arr, 3, 0x100000, nbytes, None)

    assert init(None) == -1 and b"layers" in lib.firp_last_error(None)
    assert init([0, 1, L + 1]) == -1 and b"outside" in lib.firp_last_error(None)
    assert init([-1, 0, 1]) == -1
    assert init([2, 1, 2]) == -1 and b"decrease" in lib.firp_last_error(None)
    assert not h.ctx
    assert init([0, 1, L]) == 0 and h.ctx
    h.close()
    assert init([1, 1, 1]) == 0 and h.ctx
    h.close()


def test_state_and_prefill_errors_leave_no_device_work(lib):
    h = _HostCtx(lib)
    assert h.init() == 0
    acc = np.zeros((2, 9), dtype=np.int32)
    n = np.zeros(2, dtype=np.int32)
    t, keep = binding.make_tree([-1, 0], [0, 0], None)
    p = binding._p
    assert lib.firp_step(h.ctx, C.byref(t), p(acc), p(n)) == -2          # step before prefill
    assert b"before firp_prefill" in lib.firp_last_error(h.ctx)
    toks = np.array([1, 2, 3], dtype=np.int32)
    first = np.zeros(2, dtype=np.int32)
    assert lib.firp_prefill(h.ctx, 3, p(toks), p(np.array([1, 1, 1], dtype=np.int32)), p(first)) == -3
    assert lib.firp_prefill(h.ctx, 1, p(toks), p(np.array([0], dtype=np.int32)), p(first)) == -1
    assert lib.firp_prefill(h.ctx, 1, p(toks), p(np.array([65], dtype=np.int32)), p(first)) == -3
    bad = np.array([1, 128, 3], dtype=np.int32)
    assert lib.firp_prefill(h.ctx, 1, p(bad), p(np.array([3], dtype=np.int32)), p(first)) == -1
    assert lib.firp_prefill(h.ctx, 1, None, p(np.array([3], dtype=np.int32)), p(first)) == -1
    assert lib.firp_step(h.ctx, C.byref(t), p(acc), p(n)) == -2          # still not prefilled
    assert lib.firp_set_option(h.ctx, b"nonsense", 1) == -1
    h.close()


def test_tree_validation(lib):
    h = _HostCtx(lib, k=2)
    assert h.init() == 0
    rows = C.c_int32(0)

    def check(parent, rank, anchor):
        t, keep = binding.make_tree(parent, rank, anchor)
        return lib.firp_check_tree(h.ctx, C.byref(t), C.byref(rows))

    assert check([-1, 0, 0, 1], [0, 0, 1, 3], [1, 0, 0, 1]) == 0 and rows.value == 4 + 2 * 2
    assert check([-1, 0, 0, 1], [0, 0, 1, 3], None) == 0 and rows.value == 4 + 2 * 4
    assert check([-1], [0], [0]) == 0 and rows.value == 1
    assert check([0, 0], [0, 0], None) == -1                         # root's parent must be -1
    assert check([-1, 1], [0, 0], None) == -1                        # parent not earlier
    assert check([-1, 2, 0], [0, 0, 0], None) == -1
    assert check([-1, 0], [0, 4], None) == -1                        # rank >= b_max
    assert check([-1, 0], [0, -1], None) == -1
    assert check([-1] + list(range(8)), [0] * 9, [0] * 9) == -3      # 9 nodes > max_nodes 8
    assert check([-1, 0, 1, 2, 3, 4, 5], [0] * 7, None) == -3        # 7 + 2*7 rows > max_rows 16
    assert check([-1, 0, 1, 2, 3, 4, 5], [0] * 7, [0] * 7) == 0 and rows.value == 7
    t = binding.Tree(0, None, None, None)
    assert lib.firp_check_tree(h.ctx, C.byref(t), None) == -1
    assert lib.firp_check_tree(h.ctx, None, None) == -1
    h.close()
    # depth limit (FIRP_MAX_K levels)
    h = _HostCtx(lib, k=0, max_nodes=12, max_rows=12)
    assert h.init() == 0
    assert check([-1] + list(range(8)), [0] * 9, None) == 0          # depth 8
    assert check([-1] + list(range(9)), [0] * 10, None) == -1        # depth 9
    h.close()
