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


def oracle_layer_case(cfg, batch0, ft_window, prefill_chunk, bwd_windows, seed=0, storage=None, dtype=np.float64):
    """The oracle's side of a whole-layer parity case, alone: forward iterations until the finetune sequence is
    through (seeded inputs as in the GPU parity tests), then its token-window backward with the same scaled
    MSE gradient.  -> {name: array} of every tensor those tests compare.  `storage` / `dtype` as in
    oracle.layer (storage rounding mode, arithmetic type)."""
    from oracle import layer as OL
    from oracle.maps import build_maps
    from workload.configs import KIND_FINETUNE
    W, lora = gen.layer_weights(cfg, seed, 0), gen.lora_weights(cfg, seed, 0)
    pool = OL.KVPool(batch0.num_pages, cfg.page_size, cfg.kv_dim, dtype=dtype)
    ft_seq = [r.seq_id for r in batch0.requests if r.kind == KIND_FINETUNE][0]
    L = batch0.seq_capacity[ft_seq]
    st = OL.FtState(cfg, L, dtype=dtype)
    for r in batch0.requests:
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            sl = pool.slots(batch0.seq_pages[r.seq_id], r.start_pos)
            pool.k[sl], pool.v[sl] = k, v
    out = {}
    batch, it = batch0, 0
    y_ft = np.zeros((L, cfg.hidden))
    while any(r.kind == KIND_FINETUNE for r in batch.requests):
        x = gen.layer_input(cfg, seed, batch.n_tokens, tag=f"x{it}")
        om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
        y = OL.layer_forward_mixed(cfg, W, lora, om, x, pool, {ft_seq: st}, dtype=dtype, storage=storage)
        out[f"y it{it}"] = np.asarray(y, dtype=np.float64)
        for r, off in zip(batch.requests, np.cumsum([0] + [q.n_new for q in batch.requests])):
            if r.kind == KIND_FINETUNE:
                y_ft[r.start_pos:r.start_pos + r.n_new] = y[off:off + r.n_new]
        batch = gen.advance(batch, prefill_chunk=prefill_chunk, ft_window=ft_window)
        it += 1
    out["y_ft"] = y_ft
    return out, (W, lora, pool, st, ft_seq, L)


def oracle_layer_case_backward(cfg, batch0, bwd_windows, seed, state, dY, storage=None, dtype=np.float64):
    """second half of oracle_layer_case: the backward windows for a given dY [L, H] -> {name: array}"""
    from oracle import layer as OL
    W, lora, pool, st, ft_seq, L = state
    slots = pool.slots(batch0.seq_pages[ft_seq], L)
    grads, dX, l = {}, np.zeros((L, cfg.hidden)), L
    for s in bwd_windows:
        dX[l - s:l] = OL.layer_backward_window(cfg, W, lora, st, pool.k[slots[:l]].astype(dtype), pool.v[slots[:l]].astype(dtype),
                                               l - s, s, dY[l - s:l], grads, dtype=dtype, storage=storage)
        l -= s
    out = {"dX": dX, "dk_accum": np.asarray(st.dk_accum, dtype=np.float64), "dv_accum": np.asarray(st.dv_accum, dtype=np.float64)}
    for name in ("q_cache", "x2", "gate", "up", "attn", "lse"):
        out["saved " + name] = np.asarray(getattr(st, name), dtype=np.float64)
    for t in cfg.lora_targets:
        out[f"dA[{t}]"], out[f"dB[{t}]"] = np.asarray(grads[t][0], dtype=np.float64), np.asarray(grads[t][1], dtype=np.float64)
    return out
