"""One co-serving iteration through a whole model: the mixed token batch goes forward through every
decoder layer (each with its own frozen weights, LoRA adapter, paged KV pool and finetune state), the
finetune window's top rows go through the generative loss head, and the window's gradient comes back
down through every layer (Alg. 2's Forward and Backward loops over the layers for one window, with the
inference tokens of Sec. 6.2 in the same batch); Adam over every bypass matrix is timed on its own,
since it runs once per finetune sequence, not once per iteration.

    python -m paper_2402_18789_amd.model_iter [--config c3|c4|c5] [--layers N] [--steps 5] [--warmup 2]

Default: the 8B-shaped model (32 layers, vocabulary 128 256) with a token budget of 2048 = 512 decode
tokens (log-normal contexts, median 1024) + 1024 prefill tokens (whole prompts of 128..1024 tokens) +
the last 512-token window of a 2048-token finetune sequence; synthetic weights and caches.  Prints one
JSON line.  c4: the 14B shape (48 layers, LoRA on all seven projections, window 1024 of 4096, half the
budget inference); c5: the 32B shape (64 layers, rank 32, T = 4096), whose weights, 64 KV pools and
finetune state fill most of the GPU's memory; --inference-share (c4) moves the split of the budget between
inference tokens and the finetune window (25 / 50 / 75 / 90 %: windows of 1536 / 1024 / 512 / 205 rows).  A measurement: parity of the same calls chained over layers is what the GPU tests check."""
import argparse
import json
import time

import numpy as np
import torch

import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH
from workload import gen
from workload.configs import CONFIGS

VOCAB = 128256
MODELS = {   # configuration, batch recipe, vocabulary
    "c3": ("c3_llama8b_full", gen.batch_c3, 128256),
    "c4": ("c4_qwen14b_full", gen.batch_c4, 152064),
    "c5": ("c5_qwen32b_full", gen.batch_c5, 152064),
}


def build(cfg, batch, n_layers, vocab, seed, host_seeded_layers=(), sample=()):
    """Device state of the whole model.  Layer 0 takes the seeded host weights; the others get weights of
    the same law from the device generator (436 MB per layer: generating them on the host would take
    longer than the measurement).  host_seeded_layers: layers whose weights and adapter are the host
    generator's for that layer index instead (so that a check can regenerate them), and in whose pools the
    cached prefixes of the requests in `sample` are the host generator's rows."""
    dt = HH.TORCH_DTYPE[cfg.dtype]
    W, lora = gen.layer_weights(cfg, seed, 0), gen.lora_weights(cfg, seed, 0)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ft_req = [r for r in batch.requests if r.kind == 2][0]
    L = batch.seq_capacity[ft_req.seq_id]
    layers, pools, fts = [], [], []
    # every bypass matrix of the model and its gradient in two flat buffers: one Adam launch, one gradient fill
    arena = HH.ParamArena(n_layers * HH.lora_param_elems(cfg), dt) if cfg.lora_targets else None
    for n in range(n_layers):
        if n > 0 and n in host_seeded_layers:
            ly = HH.DeviceLayer(cfg, gen.layer_weights(cfg, seed, n), gen.lora_weights(cfg, seed, n), arena=arena)
        else:
            ly = HH.DeviceLayer(cfg, W, lora, arena=arena)
        if n > 0 and n not in host_seeded_layers:
            for name in ("wqkv", "wo", "wgu", "wd"):
                t = ly.t[name]
                t.copy_((0.02 * torch.randn(t.shape, generator=g, device="cuda", dtype=torch.float32)).to(dt))
            for t in cfg.lora_targets:
                ly.A[t].copy_((0.02 * torch.randn(ly.A[t].shape, generator=g, device="cuda")).to(dt))
                ly.Bm[t].copy_((0.01 * torch.randn(ly.Bm[t].shape, generator=g, device="cuda")).to(dt))
        pool = HH.DevicePool(cfg, batch.num_pages)
        pool.fill_random(seed + n)
        if n in host_seeded_layers:
            for r in sample:
                if r.start_pos:
                    k, v = gen.kv_prefix(cfg, seed, n, r.seq_id, r.start_pos)
                    pool.write_rows(batch.seq_pages[r.seq_id], k, v)
        layers.append(ly)
        pools.append(pool)
        fts.append(HH.DeviceFtState(cfg, L))
        print("  layer %d of %d resident (%.1f GB allocated)" % (n + 1, n_layers, torch.cuda.memory_allocated() / 1e9), flush=True)
    gain = torch.ones(cfg.hidden, device="cuda", dtype=dt)
    w_lm = (0.02 * torch.randn((vocab, cfg.hidden), generator=g, device="cuda", dtype=torch.float32)).to(dt)
    return layers, pools, fts, gain, w_lm, ft_req, L, arena


def run(n_layers=None, steps=5, warmup=2, seed=0, vocab=None, model="c3", inference_share=None, capture_layers=(),
        sample=()):
    """capture_layers: layers whose input rows, output rows, incoming gradient and outgoing gradient of the LAST
    timed iteration are kept (copies on the device) and returned under "captured" together with the layers'
    device objects, for a caller that checks sampled layers of the whole-model run one by one; those layers are
    built host-seeded (see build), with the cached prefixes of `sample`'s requests."""
    cfg_name, make_batch, model_vocab = MODELS[model]
    cfg = CONFIGS[cfg_name]
    n_layers = n_layers or cfg.n_layers
    vocab = vocab or model_vocab
    batch = make_batch(seed) if inference_share is None else make_batch(seed, inference_share)
    dt = HH.TORCH_DTYPE[cfg.dtype]
    layers, pools, fts, gain, w_lm, ft_req, L, arena = build(cfg, batch, n_layers, vocab, seed, tuple(capture_layers), sample)
    captured = {n: {} for n in capture_layers}
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    hm = db.host_maps
    T, n_ft = hm.T, hm.n_ft
    ws = HH.Workspace(layers[0].c, T, hm.n_parts, n_ft, L)
    head = B.LmHead(cfg.hidden, vocab, HH.DTYPE_CODE[cfg.dtype], cfg.rms_eps, gain.data_ptr(), w_lm.data_ptr())
    hb = B.flexco_lm_loss_workspace_bytes(head, n_ft)
    hws = torch.empty(hb, dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    g = gen.rng(seed, "model_iter", "targets")
    targets = torch.from_numpy(g.integers(0, vocab, n_ft).astype(np.int32)).to("cuda")
    x0 = torch.from_numpy(gen.layer_input(cfg, seed, T)).to("cuda", dt)
    xa, xb = torch.empty_like(x0), torch.empty_like(x0)
    da, dbuf = torch.empty((n_ft, cfg.hidden), dtype=dt, device="cuda"), torch.empty((n_ft, cfg.hidden), dtype=dt, device="cuda")
    ft_off = int(np.cumsum([0] + [r.n_new for r in batch.requests])[batch.requests.index(ft_req)])
    pages = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]

    # the library's own loop over the layers (one call per pass); with capture_layers the per-layer calls, so that
    # a layer's input and output can be copied in between
    model_arr, model_keep = B.make_model_layers([(layers[n].w, layers[n].lora, pools[n].c, fts[n].c) for n in range(n_layers)])

    def reset():
        # the window's accumulator rows start from zero (a sequence's last window: nothing above it), and
        # so do the gradients; the caller's business between iterations, outside the timed bracket
        for ft in fts:
            ft.zero_accum()
        if arena is not None:
            arena.grad.zero_()
        else:
            for ly in layers:
                ly.zero_grads()
        loss.zero_()

    def iteration(timed):
        if timed:
            ev[0].record()
        if captured:
            src = x0
            for n in range(n_layers):
                dst = xa if n % 2 == 0 else xb
                B.flexco_layer_forward(layers[n].c, layers[n].w, layers[n].lora, db.maps, src, dst, pools[n].c, fts[n].c, ws.ptr, ws.bytes)
                if timed and n in captured:
                    captured[n]["x_in"], captured[n]["x_out"] = src.clone(), dst.clone()
                src = dst
        else:
            B.flexco_model_forward(layers[0].c, model_arr, n_layers, db.maps, x0, xa, xb, ws.ptr, ws.bytes)
            src = xa
        if timed:
            ev[1].record()
        top = src[ft_off:ft_off + n_ft]
        B.flexco_lm_loss(head, top, targets, n_ft, 1.0 / L, loss, da, hws, hb)
        if timed:
            ev[2].record()
        if captured:
            dcur, dnext = da, dbuf
            for n in range(n_layers - 1, -1, -1):
                B.flexco_lora_bwd(layers[n].c, layers[n].w, layers[n].lora, pools[n].c, pages, len(pages), fts[n].c,
                                  ft_req.start_pos, ft_req.n_new, dcur, dnext if n > 0 else None, ws.ptr, ws.bytes)
                if timed and n in captured:
                    captured[n]["dY"], captured[n]["dX"] = dcur.clone(), (dnext.clone() if n > 0 else None)
                dcur, dnext = dnext, dcur
        else:
            B.flexco_model_backward(layers[0].c, model_arr, n_layers, pages, len(pages), ft_req.start_pos, ft_req.n_new, da,
                                    dbuf, False, ws.ptr, ws.bytes)
        if timed:
            ev[3].record()
        return src

    for _ in range(warmup):
        reset()
        iteration(False)
    torch.cuda.synchronize()
    wall, phases = [], []
    for _ in range(steps):
        reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = iteration(True)
        torch.cuda.synchronize()
        wall.append((time.perf_counter() - t0) * 1e3)
        phases.append([ev[i].elapsed_time(ev[i + 1]) for i in range(3)])
    ph = np.median(np.asarray(phases), axis=0)
    ms = float(np.median(wall))
    finite = bool(torch.isfinite(out.float()).all().item()) and bool(torch.isfinite(loss).item())
    grad_norm = float(sum(layers[n].dB[t].double().pow(2).sum().item() for n in range(n_layers) for t in cfg.lora_targets) ** 0.5)

    # Adam over every bypass matrix of the model (fp32 master copy of the bf16 parameters), once per sequence:
    # one call over the flat parameter buffer
    adam_ms, adam_launches = [], 0
    if arena is not None:
        n_par = arena.used
        master = arena.param[:n_par].float()
        m1, m2 = torch.zeros(n_par, dtype=torch.float32, device="cuda"), torch.zeros(n_par, dtype=torch.float32, device="cuda")
        for k in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.flexco_adam_step(arena.param, master, arena.grad, m1, m2, n_par, HH.DTYPE_CODE[cfg.dtype], 1e-4, 0.9, 0.999, 1e-8, k + 1)
            torch.cuda.synchronize()
            adam_ms.append((time.perf_counter() - t0) * 1e3)
        adam_launches = 1
    positions = int(sum(r.start_pos + r.n_new for r in batch.requests))
    p_layer = (cfg.q_dim + 2 * cfg.kv_dim) * cfg.hidden + cfg.q_dim * cfg.hidden + 3 * cfg.hidden * cfg.ffn
    extra = {}
    if capture_layers:
        extra["captured"] = {"rows": captured, "layers": layers, "fts": fts, "batch": batch, "ft_req": ft_req, "seq_len": L,
                             "cfg": cfg}
    return {
        **extra,
        "what": "one co-serving iteration through the whole model: forward of the mixed batch through every layer, "
                "loss head on the finetune window, the window's backward through every layer",
        "config": {"workload": cfg_name, "layers": n_layers, "tokens": T, "finetune_tokens": n_ft, "requests": hm.n_req,
                   "cached_positions": positions, "vocab": vocab},
        "ms_per_iteration": ms, "tokens_per_s": T / ms * 1e3, "finetune_tokens_per_s": n_ft / ms * 1e3,
        "forward_ms": float(ph[0]), "loss_head_ms": float(ph[1]), "backward_ms": float(ph[2]),
        "ms_per_layer": (float(ph[0]) + float(ph[2])) / n_layers,
        "adam_ms_once_per_sequence": float(np.median(adam_ms)) if adam_ms else 0.0, "adam_launches": adam_launches,
        "layer_loop": "per-layer calls (capture)" if captured else "flexco_model_forward / flexco_model_backward",
        "resident_gb": {"weights": n_layers * p_layer * 2 / 1e9, "kv_pools": n_layers * batch.num_pages * cfg.page_size * 2 * cfg.kv_dim * 2 / 1e9,
                        "allocated": torch.cuda.memory_allocated() / 1e9},
        "loss": float(loss.item()), "lora_grad_norm_dB": grad_norm, "finite": finite,
        "dtype": cfg.dtype, "data": "synthetic",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", choices=sorted(MODELS), default="c3")
    ap.add_argument("--layers", type=int, default=0, help="0 = the model's own number of layers")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--inference-share", type=float, default=None,
                    help="c4 only: share of the 2048-token budget that is inference tokens (0.25, 0.5, 0.75, 0.9)")
    a = ap.parse_args()
    if a.inference_share is not None and a.config != "c4":
        ap.error("--inference-share belongs to --config c4")
    print(json.dumps(run(a.layers, a.steps, a.warmup, a.seed, model=a.config, inference_share=a.inference_share)))


if __name__ == "__main__":
    main()
