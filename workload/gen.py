"""Seeded input generators shared by the oracle-side and HIP-side harnesses.

Everything here is either random data (counter-based Philox streams keyed by a
base seed and a tensor name, so any tensor can be regenerated on its own) or the
description of a mixed batch (which requests, how long, which physical pages).
No method arithmetic lives here.

Input recipe (stands in for the paper's ShareGPT / BurstGPT / Sky-T1 workloads of
Sec. 8, which are not available offline):
  * base weights ~ N(0, 0.02), RMSNorm gains 1 + N(0, 0.02), QKV bias ~ N(0, 0.02)
  * LoRA A ~ N(0, 0.02), B ~ N(0, 0.01)
  * layer inputs, cached K/V prefixes and loss targets ~ N(0, 1)
  * values are rounded to the configuration's storage type, so both sides see
    identical numbers
  * pages: lowest-free-id allocation in seq_id order, then a seeded permutation
    of physical page ids (models a fragmented pool)
"""
import zlib
from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np

from .configs import (LayerCfg, Request, TARGETS, target_dims, KIND_DECODE, KIND_PREFILL,
                      KIND_FINETUNE)


def rng(seed: int, *names) -> np.random.Generator:
    """Independent Philox stream for (seed, names...)."""
    key = zlib.crc32("/".join(str(n) for n in names).encode())
    return np.random.Generator(np.random.Philox(key=[(seed << 32) | key, 0x9E3779B97F4A7C15]))


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bfloat16
    (round to nearest, ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def storage_round(cfg: LayerCfg, a: np.ndarray) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    return round_bf16(a) if cfg.dtype == "bf16" else a


def normal(cfg, g, shape, std=1.0, mean=0.0):
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return storage_round(cfg, a)


def layer_weights(cfg: LayerCfg, seed: int, layer: int = 0) -> Dict[str, np.ndarray]:
    """Frozen base weights of one decoder layer, each [out_features, in_features]."""
    H, F = cfg.hidden, cfg.ffn
    shapes = {"wq": (cfg.q_dim, H), "wk": (cfg.kv_dim, H), "wv": (cfg.kv_dim, H),
              "wo": (H, cfg.q_dim), "wg": (F, H), "wu": (F, H), "wd": (H, F)}
    w = {}
    for name, shp in shapes.items():
        w[name] = normal(cfg, rng(seed, cfg.name, layer, name), shp, std=0.02)
    for name in ("g1", "g2"):
        w[name] = normal(cfg, rng(seed, cfg.name, layer, name), (H,), std=0.02, mean=1.0)
    if cfg.qkv_bias:
        for name, n in (("bq", cfg.q_dim), ("bk", cfg.kv_dim), ("bv", cfg.kv_dim)):
            w[name] = normal(cfg, rng(seed, cfg.name, layer, name), (n,), std=0.02)
    return w


def lora_weights(cfg: LayerCfg, seed: int, layer: int = 0, adapter: int = 0, b_std=0.01):
    """LoRA matrices per target: A [in, r], B [r, out]."""
    out = {}
    for t in cfg.lora_targets:
        din, dout = target_dims(cfg, t)
        A = normal(cfg, rng(seed, cfg.name, layer, "loraA", adapter, t), (din, cfg.lora_rank), std=0.02)
        B = normal(cfg, rng(seed, cfg.name, layer, "loraB", adapter, t), (cfg.lora_rank, dout), std=b_std)
        out[t] = (A, B)
    return out


def ia3_weights(cfg: LayerCfg, seed: int, layer: int = 0, adapter: int = 0, std=0.25):
    """(IA)^3 scaling vectors {"k", "v": [kv_dim], "ff": [ffn]}, 1 + N(0, std) in the storage type (the
    method starts them at one; a trained adapter has moved away from it, so that a dropped scale shows)."""
    return {name: normal(cfg, rng(seed, cfg.name, layer, "ia3", adapter, name), (n,), std=std, mean=1.0)
            for name, n in (("k", cfg.kv_dim), ("v", cfg.kv_dim), ("ff", cfg.ffn))}


def layer_input(cfg: LayerCfg, seed: int, T: int, tag="x") -> np.ndarray:
    return normal(cfg, rng(seed, cfg.name, tag), (T, cfg.hidden))


def kv_prefix(cfg: LayerCfg, seed: int, layer: int, seq_id: int, n: int):
    """Seeded cached (K, V) rows [n, kv_dim] of a sequence prefix, to be read as the
    post-RoPE keys and the values the earlier iterations wrote."""
    g = rng(seed, cfg.name, layer, "kvprefix", seq_id)
    kv = g.standard_normal((2, n, cfg.kv_dim), dtype=np.float32)
    kv = storage_round(cfg, kv)
    return kv[0], kv[1]


def loss_targets(cfg: LayerCfg, seed: int, L: int) -> np.ndarray:
    return normal(cfg, rng(seed, cfg.name, "targets"), (L, cfg.hidden))


@dataclass
class Batch:
    requests: List[Request]
    seq_pages: Dict[int, np.ndarray]      # seq_id -> int32 physical page ids
    seq_capacity: Dict[int, int]          # seq_id -> tokens the page list can hold
    num_pages: int
    page_size: int

    @property
    def n_tokens(self):
        return sum(r.n_new for r in self.requests)

    @property
    def n_ft_tokens(self):
        return sum(r.n_new for r in self.requests if r.kind == KIND_FINETUNE)


def allocate_pages(capacities: Dict[int, int], page_size: int, seed: int, slack_pages: int = 3,
                   permute: bool = True):
    """Lowest-free-id page allocation in seq_id order, then a seeded permutation of
    the physical ids over a pool with slack_pages unused pages."""
    nxt = 0
    lists = {}
    for sid in sorted(capacities):
        n = -(-capacities[sid] // page_size)
        lists[sid] = np.arange(nxt, nxt + n, dtype=np.int64)
        nxt += n
    num_pages = nxt + slack_pages
    if permute:
        perm = rng(seed, "pageperm", num_pages).permutation(num_pages)
    else:
        perm = np.arange(num_pages)
    return {sid: perm[l].astype(np.int32) for sid, l in lists.items()}, num_pages


def mixed_batch(page_size, seed, decode_ctx=(), prefill=(), finetune=(), permute=True,
                ft_adapter=0, extra_capacity=0) -> Batch:
    """decode_ctx: context length of each decode request INCLUDING the new token.
    prefill / finetune: tuples (start_pos, n_new, total_len).
    Token order in the batch: decode, then prefill chunks, then finetune windows."""
    reqs, caps = [], {}
    sid = 0
    for ctx in decode_ctx:
        reqs.append(Request(KIND_DECODE, sid, int(ctx) - 1, 1, -1))
        caps[sid] = int(ctx) + extra_capacity
        sid += 1
    for (start, n_new, total) in prefill:
        reqs.append(Request(KIND_PREFILL, sid, int(start), int(n_new), -1))
        caps[sid] = int(total)
        sid += 1
    for (start, n_new, total) in finetune:
        reqs.append(Request(KIND_FINETUNE, sid, int(start), int(n_new), ft_adapter))
        caps[sid] = int(total)
        sid += 1
    pages, num_pages = allocate_pages(caps, page_size, seed, permute=permute)
    return Batch(reqs, pages, caps, num_pages, page_size)


def with_adapters(batch: Batch, ids) -> Batch:
    """The same batch with the inference requests served by different adapters: request i (finetune
    requests aside) gets ids[i % len(ids)] (-1: base model only)."""
    reqs = [r if r.kind == KIND_FINETUNE else Request(r.kind, r.seq_id, r.start_pos, r.n_new, int(ids[i % len(ids)]))
            for i, r in enumerate(batch.requests)]
    return Batch(reqs, batch.seq_pages, batch.seq_capacity, batch.num_pages, batch.page_size)


def advance(batch: Batch, prefill_chunk=None, ft_window=None) -> Batch:
    """The next iteration of the same sequences: every decode request moves on one
    token; prefill / finetune requests continue with the given chunk / window
    length (dropped when None or when the sequence is complete)."""
    reqs = []
    for r in batch.requests:
        nxt = r.start_pos + r.n_new
        cap = batch.seq_capacity[r.seq_id]
        if r.kind == KIND_DECODE:
            if nxt < cap:
                reqs.append(Request(r.kind, r.seq_id, nxt, 1, r.adapter))
        else:
            n = prefill_chunk if r.kind == KIND_PREFILL else ft_window
            if n and nxt < cap:
                reqs.append(Request(r.kind, r.seq_id, nxt, min(n, cap - nxt), r.adapter))
    return Batch(reqs, batch.seq_pages, batch.seq_capacity, batch.num_pages, batch.page_size)


# ---------------------------------------------------------------------------
# The named workloads.
# ---------------------------------------------------------------------------

def batch_c1(seed=0) -> Batch:
    """Tiny fp32 case: 4 decode tokens (contexts 16, 32, 48, 64), one prefill chunk
    of 32 of a 64-token prompt, one finetune sequence of 64 taken in windows of 32."""
    return mixed_batch(16, seed, decode_ctx=(16, 32, 48, 64), prefill=[(0, 32, 64)],
                       finetune=[(0, 32, 64)], extra_capacity=2)


def batch_c2(seed=0) -> Batch:
    """8B-shaped single-layer case, token budget 1024: 256 decode tokens (contexts
    uniform in 512..4096), two prefill chunks of 256 (one with no prefix, one at
    offset 768 of a 1024-token prompt) and the last 256-token window of a
    2048-token finetune sequence."""
    ctx = rng(seed, "c2", "decode_ctx").integers(512, 4097, size=256)
    return mixed_batch(16, seed, decode_ctx=ctx, prefill=[(0, 256, 256), (768, 256, 1024)],
                       finetune=[(1792, 256, 2048)])


def batch_c3(seed=0) -> Batch:
    """8B-shaped whole-model case, token budget 2048: 512 decode tokens whose contexts follow a
    log-normal law (median 1024, sigma 0.8, clipped to 16..8192), 1024 prefill tokens made of whole
    prompts with lengths uniform in 128..1024 (the last one cut to the budget) and the last 512-token
    window of a 2048-token finetune sequence."""
    g = rng(seed, "c3", "lengths")
    ctx = np.clip(np.round(np.exp(g.normal(np.log(1024.0), 0.8, size=512))), 16, 8192).astype(int)
    prefill, left = [], 1024
    while left > 0:
        n = int(min(left, g.integers(128, 1025)))
        prefill.append((0, n, n))
        left -= n
    return mixed_batch(16, seed, decode_ctx=ctx, prefill=prefill, finetune=[(1536, 512, 2048)])


def _lognormal_lengths(g, n, median, sigma, lo, hi):
    return np.clip(np.round(np.exp(g.normal(np.log(float(median)), sigma, size=n))), lo, hi).astype(int)


def _whole_prompts(g, budget, lo=128, hi=1024):
    prefill, left = [], budget
    while left > 0:
        n = int(min(left, g.integers(lo, hi + 1)))
        prefill.append((0, n, n))
        left -= n
    return prefill


C4_SHARES = (0.25, 0.5, 0.75, 0.9)


def batch_c4(seed=0, inference_share=0.5) -> Batch:
    """14B-shaped whole-model case, token budget 2048 at an inference share of 25 / 50 / 75 / 90 %: the inference
    tokens (512 / 1024 / 1536 / 1843) are half decode tokens (contexts log-normal, median 1024 - 768 at 90 % -,
    sigma 0.8, clipped to 16..8192) and half prefill tokens as whole prompts; the rest of the budget (1536 / 1024 / 512 /
    205 tokens) is the last window of a 4096-token finetune sequence."""
    budget, L = 2048, 4096
    n_inf = int(budget * inference_share)
    n_dec = n_inf // 2
    n_ft = budget - n_inf
    assert 0 < n_ft <= L and n_dec > 0
    g = rng(seed, "c4", "lengths") if inference_share == 0.5 else rng(seed, "c4", "lengths", n_inf)
    # 921 decode requests at the law's median of 1024 would hold 1.3 M cached positions: 254 GB of cache over the
    # model's 48 layers, more than one GPU has beside the weights; the 90 % point takes a median of 768
    median = 1024 if n_dec <= 768 else 768
    ctx = _lognormal_lengths(g, n_dec, median, 0.8, 16, 8192)
    return mixed_batch(16, seed, decode_ctx=ctx, prefill=_whole_prompts(g, n_inf - n_dec), finetune=[(L - n_ft, n_ft, L)])


def batch_c5(seed=0) -> Batch:
    """32B-shaped whole-model case, token budget 4096: 1024 decode tokens (contexts log-normal, median 320,
    sigma 1.0, clipped to 16..16384: the law's scale is what lets 64 layers of cache, the weights and the
    finetune state share one GPU's memory), 2048 prefill tokens as whole prompts, and the last 1024-token
    window of a 4096-token finetune sequence."""
    g = rng(seed, "c5", "lengths")
    ctx = _lognormal_lengths(g, 1024, 320, 1.0, 16, 16384)
    return mixed_batch(16, seed, decode_ctx=ctx, prefill=_whole_prompts(g, 2048), finetune=[(3072, 1024, 4096)])


def batch_scaled(seed, n_decode, ctx_lo, ctx_hi, prefill, finetune, page_size=16) -> Batch:
    """Reduced-size batch of the same structure as batch_c2 (parity tests)."""
    ctx = rng(seed, "scaled", "decode_ctx", n_decode, ctx_lo, ctx_hi).integers(ctx_lo, ctx_hi + 1, size=n_decode)
    return mixed_batch(page_size, seed, decode_ctx=ctx, prefill=prefill, finetune=finetune)


def sample_requests(batch: Batch, n_decode: int):
    """A bounded sample of a batch's requests for checks the oracle runs one by one: the first
    n_decode decode requests, the first and the last prefill request (the benchmark batch's two chunks: the one
    without a cached prefix and the one behind 768 cached positions; in the whole-model batches a whole prompt
    and the truncated last one) and the finetune window."""
    dec = [r for r in batch.requests if r.kind == KIND_DECODE][:n_decode]
    pre = [r for r in batch.requests if r.kind == KIND_PREFILL]
    pre = pre[:1] + pre[-1:] if len(pre) > 1 else pre
    ftr = [r for r in batch.requests if r.kind == KIND_FINETUNE]
    return dec + pre + ftr


def sample_token_rows(batch: Batch, sample):
    """Token indices (in the full batch) of the sampled requests, in sample order."""
    tok_off = np.cumsum([0] + [r.n_new for r in batch.requests])
    idx = {id(r): i for i, r in enumerate(batch.requests)}
    return np.concatenate([np.arange(tok_off[idx[id(r)]], tok_off[idx[id(r)] + 1]) for r in sample])
