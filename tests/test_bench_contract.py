"""Host-side checks of bench.py: the one-GPU rule and the algorithmic byte count it divides by."""
import os
import subprocess
import sys

import pytest

from paper_2410_20488_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be mistaken for a measurement


def test_algorithmic_bytes_of_the_13b_step():
    """Every weight once, the live cache once, the step rows' K/V out and in, written out by hand for
    the LLaMA-2-13B shapes with k = 3 maps at layer 20, 64 nodes, 67 rows above the maps, 1100 cached
    tokens: 317.19 M parameters per layer, 800 KiB of cache per token over the 40 layers."""
    cfg = synth.CONFIGS["13b"]
    per_layer = 4 * 5120 * 5120 + 3 * 5120 * 13824
    assert cfg.layer_params() == per_layer == 317_194_240
    weights = 2 * (40 * per_layer + 32000 * 5120 + 3 * 5120 * 5120)
    kv_row = 2 * 40 * 128 * 2                          # K and V of one row in one layer, bf16
    assert kv_row * 40 == 800 * 1024
    cache = 1100 * kv_row * 40
    step_rows = 2 * kv_row * (64 * 20 + 67 * 20)
    assert bench.algorithmic_bytes(cfg, 64, 67, 1100) == pytest.approx(weights + cache + step_rows, rel=1e-12)
    assert 26.7e9 < weights + cache + step_rows < 26.9e9
    # four sequences move four caches and four sets of step rows past one set of weights
    assert bench.algorithmic_bytes(cfg, 64, 67, 1100, batch=4) == pytest.approx(weights + 4 * (cache + step_rows))
    # one prediction layer per step: pseudo row i exists from layer t_i on
    import dataclasses
    stag = dataclasses.replace(cfg, firp_layers=(25, 30, 35))
    rows = 64 * 25 + 65 * 5 + 66 * 5 + 67 * 5
    assert bench.algorithmic_bytes(stag, 64, 67, 1100) == pytest.approx(weights + cache + 2 * kv_row * rows)
