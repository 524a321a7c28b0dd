#!/usr/bin/env python3
"""Benchmark of one co-serving layer iteration on one MI355X.

A step = the whole hot path on one synthetic mixed batch of the 8B-shaped single-layer
configuration: flexco_layer_forward over all 1024 tokens (256 decode tokens with contexts
uniform in 512..4096, two prefill chunks of 256, the last 256-token window of a 2048-token
finetune sequence) followed by flexco_lora_bwd of that finetune window.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--weight-copies", type=int, default=3,
                    help="independent copies of the layer weights cycled between steps, so that the "
                         "436 MB weight set is never served from the 256 MB last-level cache")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-decode", type=int, default=16)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives, no sharding); got --gpus %d" % args.gpus)
        sys.exit(2)

    import torch
    from workload import gen, CONFIGS
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = CONFIGS["c2_llama8b_layer"]
    seed = args.seed
    t_setup = time.time()
    batch = gen.batch_c2(seed)
    W = gen.layer_weights(cfg, seed, 0)
    lora = gen.lora_weights(cfg, seed, 0)
    layers = [HH.DeviceLayer(cfg, W, lora) for _ in range(max(1, args.weight_copies))]
    pool = HH.DevicePool(cfg, batch.num_pages)
    # cached prefixes: N(0,1) values for every page (device generator), then the sampled sequences the
    # CPU baseline also reads are overwritten with the host generator's rows
    pool.fill_random(seed)
    ft_req = [r for r in batch.requests if r.kind == 2][0]
    L = batch.seq_capacity[ft_req.seq_id]
    sample = gen.sample_requests(batch, args.cpu_sample_decode)
    for r in sample:
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            pool.write_rows(batch.seq_pages[r.seq_id], k, v)
    ft = HH.DeviceFtState(cfg, L)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    hm = db.host_maps
    T, n_ft = hm.T, hm.n_ft
    ws = HH.Workspace(layers[0].c, T, hm.n_parts, n_ft, L)
    x_np = gen.layer_input(cfg, seed, T)
    x = torch.from_numpy(x_np).to("cuda", torch.bfloat16)
    y = torch.empty_like(x)
    dY = torch.from_numpy(gen.layer_input(cfg, seed, n_ft, tag="dy")).to("cuda", torch.bfloat16)
    dX = torch.empty_like(dY)
    ft_pages = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")
    n_ft_pages = int(ft_pages.numel())
    log("setup %.1fs: T=%d (ft %d), requests=%d, pages=%d, attention items=%d" %
        (time.time() - t_setup, T, n_ft, hm.n_req, batch.num_pages, hm.n_items))

    def step(i):
        ly = layers[i % len(layers)]
        B.flexco_layer_forward(ly.c, ly.w, ly.lora, db.maps, x, y, pool.c, ft.c, ws.ptr, ws.bytes)
        B.flexco_lora_bwd(ly.c, ly.w, ly.lora, pool.c, ft_pages, n_ft_pages, ft.c, ft_req.start_pos, ft_req.n_new,
                          dY, dX, ws.ptr, ws.bytes)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- which kernel class dominates?  a short pass with every class timed --------------------
    probe_steps = 3
    for name, kid in B.KERNEL_IDS.items():
        B.flexco_kernel_timer_start(kid, 64 * probe_steps)
    for i in range(probe_steps):
        step(i)
    torch.cuda.synchronize()
    breakdown = {}
    for name, kid in B.KERNEL_IDS.items():
        ms, n = B.flexco_kernel_timer_stop(kid)
        breakdown[name] = {"ms_per_step": ms / probe_steps, "launches_per_step": n / probe_steps}
    dominant = max(breakdown, key=lambda k: breakdown[k]["ms_per_step"])
    log("per-step kernel classes (ms): " + ", ".join("%s=%.3f" % (k, v["ms_per_step"]) for k, v in breakdown.items()))

    # ---- the timed region: K steps, with the dominant class bracketed by events -----------------
    B.flexco_kernel_timer_start(B.KERNEL_IDS[dominant], 64 * args.steps)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    dom_ms, dom_launches = B.flexco_kernel_timer_stop(B.KERNEL_IDS[dominant])
    ms_per_step = max(wall_ms, gpu_ms) / args.steps
    value = T / (ms_per_step * 1e-3)

    roofline = roofline_for(dominant, dom_ms, dom_launches, args.steps, cfg, batch, hm)
    out = {
        "metric": "co-served tokens/s per layer iteration",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c2_llama8b_layer: 1 LLaMA-3.1-8B-shaped layer, T=1024 = 256 decode (ctx U[512,4096], "
                               "page 16) + 2x256 prefill + 256 finetune (last window of 2048); forward of all "
                               "tokens + LoRA r16 (q,k,v,o,down) window backward",
                   "tokens": T, "finetune_tokens": n_ft, "requests": hm.n_req,
                   "cached_positions": int(sum(r.start_pos + r.n_new for r in batch.requests)),
                   "weight_copies_cycled": len(layers)},
        "roofline": roofline,
        "kernel_classes_ms_per_step": {k: round(v["ms_per_step"], 4) for k, v in breakdown.items()},
        "gpu_event_ms_per_step": gpu_ms / args.steps,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, batch, sample, W, lora, seed, x_np, ft_req, L)
    print(json.dumps(out), flush=True)


def roofline_for(dominant, dom_ms, dom_launches, steps, cfg, batch, hm):
    """Algorithmic work of the dominant kernel class per launch / its measured mean duration."""
    H, F = cfg.hidden, cfg.ffn
    qd, kd = cfg.q_dim, cfg.kv_dim
    T, n_ft = hm.T, hm.n_ft
    avg_ms = dom_ms / max(1, dom_launches)
    if dominant == "attn_fwd":
        # every cached position visible to a token group is read once per kv head: K row + V row, bf16.
        # decode: contexts; chunks: each tile of tile_tokens tokens reads [0, last position of the tile]
        bytes_ = 0
        for r in batch.requests:
            if r.kind == 0:
                bytes_ += (r.start_pos + 1) * 2 * kd * 2
        decode_bytes = bytes_
        # prefill / finetune tiles re-read their prefix per tile: algorithmic minimum is once per request
        for r in batch.requests:
            if r.kind != 0:
                bytes_ += (r.start_pos + r.n_new) * 2 * kd * 2
        per_launch = bytes_
        ach = per_launch / (avg_ms * 1e-3) / 1e9
        return {"kernel": "attn_fwd_mfma_kernel", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None, "avg_launch_ms": avg_ms,
                "algorithmic_bytes_per_launch": per_launch, "decode_kv_bytes": decode_bytes,
                "launches_per_step": dom_launches / steps}
    if dominant in ("gemm_fwd", "gemm_bwd"):
        p_base = (qd + 2 * kd) * H + qd * H + 3 * H * F
        rows = T if dominant == "gemm_fwd" else n_ft
        flops_step = 2.0 * p_base * rows
        per_launch = flops_step * steps / max(1, dom_launches)
        ach = per_launch / (avg_ms * 1e-3) / 1e12
        return {"kernel": "gemm_bf16_kernel (%s)" % dominant, "bound": "mfma", "achieved": ach,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                "avg_launch_ms": avg_ms, "algorithmic_flops_per_launch": per_launch,
                "launches_per_step": dom_launches / steps}
    if dominant == "attn_bwd":
        l = max(r.start_pos + r.n_new for r in batch.requests if r.kind == 2)
        s = n_ft
        # 5 products of [s x l(avg visible)] x d per head, causal inside the window
        vis = s * (l - s) + s * (s + 1) / 2
        flops = 10.0 * cfg.n_q_heads * cfg.head_dim * vis
        ach = flops / (avg_ms * 1e-3) / 1e12
        return {"kernel": "attention window backward", "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "avg_launch_ms": avg_ms,
                "algorithmic_flops_per_launch": flops, "launches_per_step": dom_launches / steps}
    return {"kernel": dominant, "bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
            "traffic": None, "avg_launch_ms": avg_ms, "launches_per_step": dom_launches / steps}


def cpu_baseline(cfg, batch, sample, W, lora, seed, x_np, ft_req, L):
    """The oracle, as it stands, on a bounded sample of the same workload (forward of the sampled
    requests' tokens + the finetune window's backward), timed on this machine's host cores."""
    from oracle import layer as OL
    from oracle.maps import build_maps
    from workload import gen
    import threadpoolctl
    t_all = time.time()
    pool = OL.KVPool(batch.num_pages, cfg.page_size, cfg.kv_dim, dtype=np.float32)
    for r in sample:
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            sl = pool.slots(batch.seq_pages[r.seq_id], r.start_pos)
            pool.k[sl], pool.v[sl] = k, v
    rows = gen.sample_token_rows(batch, sample)
    om = build_maps(sample, batch.seq_pages, batch.page_size, batch.num_pages)
    st = {ft_req.seq_id: OL.FtState(cfg, L)}
    threads = sum(p.get("num_threads", 0) for p in threadpoolctl.threadpool_info() if p.get("user_api") == "blas") or os.cpu_count()
    log("cpu baseline: oracle on %d sampled tokens (%d requests), %d BLAS threads" % (len(rows), len(sample), threads))
    t0 = time.perf_counter()
    OL.layer_forward_mixed(cfg, W, lora, om, x_np[rows], pool, st)
    t_f = time.perf_counter() - t0
    dY = gen.layer_input(cfg, seed, ft_req.n_new, tag="dy")
    sl = pool.slots(batch.seq_pages[ft_req.seq_id], L)
    t0 = time.perf_counter()
    OL.layer_backward_window(cfg, W, lora, st[ft_req.seq_id], pool.k[sl].astype(np.float64), pool.v[sl].astype(np.float64),
                             ft_req.start_pos, ft_req.n_new, dY, {})
    t_b = time.perf_counter() - t0
    log("cpu baseline: forward %.1fs, backward %.1fs, total incl. setup %.1fs" % (t_f, t_b, time.time() - t_all))
    return {"value": len(rows) / (t_f + t_b), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d of 1024 tokens: %d decode requests, one 256-token prefill chunk, the 256-token finetune "
                      "window (forward) + that window's backward; numpy fp64" % (len(rows), len(sample) - 2),
            "seconds": t_f + t_b, "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
