"""Shared test helpers: build an oracle from a synthetic config."""
import torch

from oracle.firp_oracle import FirpOracle
from paper_2410_20488_amd import synth


def cpu_weights(weights):
    """Copy a weight dict (tensors / lists of tensors / None) to host memory."""
    out = {}
    for k, v in weights.items():
        if v is None:
            out[k] = None
        elif isinstance(v, (list, tuple)):
            out[k] = [t.detach().cpu() for t in v]
        else:
            out[k] = v.detach().cpu()
    return out


def make_oracle(cfg: synth.ModelConfig, weights, dtype=torch.float32, b_max=8, kv_round=None):
    if kv_round is None:
        kv_round = cfg.dtype == "bf16"
    return FirpOracle(n_layers=cfg.n_layers, d_model=cfg.d_model, n_q_heads=cfg.n_q_heads,
                      n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, d_ffn=cfg.d_ffn,
                      vocab=cfg.vocab, rms_eps=cfg.rms_eps, rope_base=cfg.rope_base,
                      weights=weights, firp_layer=cfg.firp_layer, k=cfg.k, b_max=b_max,
                      dtype=dtype, kv_round_bf16=kv_round, firp_layers=cfg.firp_layers)


MICRO = synth.ModelConfig("micro", 3, 64, 4, 2, 16, 96, 128, firp_layer=1, k=2, dtype="f32",
                          rms_eps=1e-6, seed=777)
