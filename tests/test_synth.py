"""The seeded input generators: determinism, distribution, tree shapes."""
import torch

from paper_2410_20488_amd import synth


def test_hash_matches_pure_python_reference():
    base = synth._i64(12345 ^ (7 << 40))
    idx = torch.arange(0, 50, dtype=torch.int64)
    got = synth._splitmix64(idx ^ base)
    for i in range(50):
        want = synth.splitmix64_py((i ^ 12345 ^ (7 << 40)) & ((1 << 64) - 1))
        assert (int(got[i]) & ((1 << 64) - 1)) == want


def test_normal_tensor_is_chunk_invariant_and_roughly_normal():
    a = synth.normal_tensor(1, 2, (1000, 37), 0.02, torch.float32)
    b = synth.normal_tensor(1, 2, (1000, 37), 0.02, torch.float32, chunk=999)
    assert torch.equal(a, b)
    assert abs(float(a.mean())) < 5e-4 and abs(float(a.std()) - 0.02) < 5e-4
    c = synth.normal_tensor(1, 3, (1000, 37), 0.02, torch.float32)
    assert not torch.equal(a, c)
    h = synth.normal_tensor(1, 2, (1000, 37), 0.02, torch.bfloat16)
    assert torch.equal(h, a.to(torch.bfloat16))


def test_prompt_tokens_in_range_and_seeded():
    t = synth.prompt_tokens(20490, 1024, 32000)
    assert t.dtype == torch.int32 and int(t.min()) >= 0 and int(t.max()) < 32000
    assert torch.equal(t, synth.prompt_tokens(20490, 1024, 32000))
    assert len(set(t.tolist())) > 900


def _check_tree(t):
    assert t.parent[0] == -1
    for v in range(1, t.n_nodes):
        assert 0 <= t.parent[v] < v
    sib = {}
    for v in range(1, t.n_nodes):
        assert (t.parent[v], t.rank[v]) not in sib
        sib[(t.parent[v], t.rank[v])] = v


def test_workload_trees():
    t = synth.workload_tree("tiny")
    assert t.parent == (-1, 0, 1, 2) and t.anchor == (1, 0, 0, 0)
    t = synth.workload_tree("7b")
    assert t.n_nodes == 41
    _check_tree(t)
    t = synth.workload_tree("13b")
    assert t.n_nodes == 64
    _check_tree(t)
    depth = [0] * 64
    for v in range(1, 64):
        depth[v] = depth[t.parent[v]] + 1
    assert [depth.count(i) for i in (1, 2, 3)] == [8, 22, 33]
    assert max(t.rank) == 7
    assert sum(synth.workload_tree("13b", "all").anchor) == 64


def test_weight_shapes_and_sizes():
    cfg = synth.CONFIGS["13b"]
    assert cfg.layer_params() == 317_194_240
    assert abs(cfg.weight_bytes() / 1e9 - 25.86) < 0.01
    w = synth.make_weights(synth.CONFIGS["tiny_gqa"], "cpu", with_bias=True)
    c = synth.CONFIGS["tiny_gqa"]
    assert w["wk"][0].shape == (c.n_kv_heads * c.head_dim, c.d_model)
    assert w["w_down"][2].shape == (c.d_model, c.d_ffn) and w["proj_b"][1].shape == (c.d_model,)
    assert w["wq"][0].dtype == torch.bfloat16
