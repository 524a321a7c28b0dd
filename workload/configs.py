"""Layer shapes and request records of the benchmark configurations.

Shapes follow the model families the paper evaluates (Sec. 8, "LLMs and PEFT
models"): LLaMA-3.1-8B and Qwen-2.5-14B/32B decoder layers with LoRA bypass
networks (Sec. 4.1).  Backbone constants the paper does not state (RMSNorm eps,
RoPE base, QKV bias) take the public values of those model families.
"""
from dataclasses import dataclass, field, replace
from typing import Tuple

# LoRA target names in bit order of the lora_targets mask (q=1, k=2, v=4, o=8,
# gate=16, up=32, down=64).
TARGETS = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass(frozen=True)
class LayerCfg:
    name: str
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    dtype: str            # "f32" | "bf16": storage type of activations, weights, caches
    rms_eps: float
    rope_theta: float
    page_size: int
    lora_rank: int
    lora_targets: Tuple[str, ...]
    lora_scale: float
    qkv_bias: bool = False
    n_layers: int = 1

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self):
        return self.q_dim + 2 * self.kv_dim

    @property
    def target_mask(self):
        return sum(1 << TARGETS.index(t) for t in self.lora_targets)

    def with_(self, **kw):
        return replace(self, **kw)


def target_dims(cfg: LayerCfg, target: str):
    """(in_features, out_features) of the base projection a LoRA target wraps."""
    return {
        "q": (cfg.hidden, cfg.q_dim),
        "k": (cfg.hidden, cfg.kv_dim),
        "v": (cfg.hidden, cfg.kv_dim),
        "o": (cfg.q_dim, cfg.hidden),
        "gate": (cfg.hidden, cfg.ffn),
        "up": (cfg.hidden, cfg.ffn),
        "down": (cfg.ffn, cfg.hidden),
    }[target]


@dataclass(frozen=True)
class Request:
    """One entry of the mixed batch: n_new tokens of sequence seq_id starting at
    absolute position start_pos (everything before start_pos is already cached)."""
    kind: int        # 0 decode, 1 prefill chunk, 2 finetune window
    seq_id: int
    start_pos: int
    n_new: int
    adapter: int     # -1: base model only; >= 0: LoRA adapter id


KIND_DECODE, KIND_PREFILL, KIND_FINETUNE = 0, 1, 2

# alpha = 2 r  ->  scale 2.0 in every configuration, so that a dropped scale shows.
CONFIGS = {
    "c1_tiny_f32": LayerCfg(
        name="c1_tiny_f32", hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688,
        dtype="f32", rms_eps=1e-5, rope_theta=10000.0, page_size=16, lora_rank=8,
        lora_targets=("q", "v", "down"), lora_scale=2.0),
    "c2_llama8b_layer": LayerCfg(
        name="c2_llama8b_layer", hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
        ffn=14336, dtype="bf16", rms_eps=1e-5, rope_theta=500000.0, page_size=16,
        lora_rank=16, lora_targets=("q", "k", "v", "o", "down"), lora_scale=2.0),
    "c3_llama8b_full": LayerCfg(
        name="c3_llama8b_full", hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
        ffn=14336, dtype="bf16", rms_eps=1e-5, rope_theta=500000.0, page_size=16,
        lora_rank=16, lora_targets=("q", "k", "v", "o", "down"), lora_scale=2.0, n_layers=32),
    "c4_qwen14b_full": LayerCfg(
        name="c4_qwen14b_full", hidden=5120, n_q_heads=40, n_kv_heads=8, head_dim=128,
        ffn=13824, dtype="bf16", rms_eps=1e-6, rope_theta=1e6, page_size=16,
        lora_rank=16, lora_targets=TARGETS, lora_scale=2.0, qkv_bias=True, n_layers=48),
    "c5_qwen32b_full": LayerCfg(
        name="c5_qwen32b_full", hidden=5120, n_q_heads=40, n_kv_heads=8, head_dim=128,
        ffn=27648, dtype="bf16", rms_eps=1e-6, rope_theta=1e6, page_size=16,
        lora_rank=32, lora_targets=TARGETS, lora_scale=2.0, qkv_bias=True, n_layers=64),
}
