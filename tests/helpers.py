"""Small shared fixtures for the oracle tests (no method arithmetic)."""
import numpy as np

from workload import LayerCfg, gen

SMALL = LayerCfg(name="small", hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn=48,
                 dtype="f32", rms_eps=1e-5, rope_theta=10000.0, page_size=4, lora_rank=4,
                 lora_targets=("q", "k", "v", "o", "gate", "up", "down"), lora_scale=2.0,
                 qkv_bias=True)


def small_layer(cfg=SMALL, seed=1, layer=0, scale_up=5.0):
    """Weights scaled up from the N(0, 0.02) recipe so that every path of a tiny layer
    carries signal well above rounding."""
    W = gen.layer_weights(cfg, seed, layer)
    W = {k: (v * scale_up if k.startswith("w") else v).astype(np.float64) for k, v in W.items()}
    lo = gen.lora_weights(cfg, seed, layer, b_std=0.02)
    lo = {t: ((A * scale_up).astype(np.float64), (B * scale_up).astype(np.float64)) for t, (A, B) in lo.items()}
    return W, lo


def rel_err(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = np.max(np.abs(b))
    return float(np.max(np.abs(a - b)) / den) if den > 0 else float(np.max(np.abs(a - b)))
