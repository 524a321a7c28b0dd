#!/usr/bin/env python3
"""Benchmark of one co-serving layer iteration on one MI355X.

A step = the whole hot path on one synthetic mixed batch of the 8B-shaped single-layer
configuration: flexco_layer_forward over all 1024 tokens (256 decode tokens with contexts
uniform in 512..4096, two prefill chunks of 256, the last 256-token window of a 2048-token
finetune sequence) followed by flexco_lora_bwd of that finetune window.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--calib-copy]
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16
KERNEL_NAMES = {"gemm_fwd": "gemm_bf16_kernel<BM,BN,false> (forward projections)",
                "gemm_bwd": "gemm_bf16_kernel<128,128,true> (input-gradient projections)",
                "attn_fwd": "attn_fwd_mfma_kernel", "attn_merge": "attn_merge_kernel",
                "attn_bwd": "attn_delta + attn_bwd_dq_mfma + attn_bwd_dkv_mfma", "elemwise": "norm/rope/swiglu/copy kernels",
                "lora": "lora_shrink/finalize/transpose/outer kernels", "generic": "type-generic fallbacks"}


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
    ap.add_argument("--cpu-sample-decode", type=int, default=32)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--overlap", action="store_true",
                    help="co-serving as in Sec. 6.2 of the paper: the window backward runs on a second stream, "
                         "concurrently with the forward of the batch, on a finetune sequence of its own")
    ap.add_argument("--no-two-stream", action="store_true", help="skip the additional two-stream measurement")
    ap.add_argument("--bypass", choices=("lora", "ia3"), default="lora",
                    help="bypass network of the finetune window: LoRA r16 on q,k,v,o,down (the headline workload) or "
                         "(IA)^3 vectors on k, v and the FFN activation (same batch, same base layer)")
    ap.add_argument("--kv-split-pages", type=int, default=0,
                    help="pages per attention work item (0 = the library's default)")
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
    use_ia3 = args.bypass == "ia3"
    if use_ia3:
        cfg = cfg.with_(lora_targets=())
    seed = args.seed
    t_setup = time.time()
    batch = gen.batch_c2(seed)
    W = gen.layer_weights(cfg, seed, 0)
    lora = None if use_ia3 else gen.lora_weights(cfg, seed, 0)
    ia3_np = gen.ia3_weights(cfg, seed, 0) if use_ia3 else None
    ia3 = HH.DeviceIa3(cfg, ia3_np) if use_ia3 else None
    layers = [HH.DeviceLayer(cfg, W, lora) for _ in range(max(1, args.weight_copies))]
    n_seq_pages = len(batch.seq_pages[[r for r in batch.requests if r.kind == 2][0].seq_id])
    pool = HH.DevicePool(cfg, batch.num_pages + n_seq_pages)   # + room for the two-stream run's own sequence
    # cached prefixes: N(0,1) values in every page (device generator); the sampled sequences the CPU
    # baseline also reads are overwritten with the host generator's rows
    pool.fill_random(seed)
    ft_req = [r for r in batch.requests if r.kind == 2][0]
    L = batch.seq_capacity[ft_req.seq_id]
    sample = gen.sample_requests(batch, args.cpu_sample_decode)
    for r in sample:
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            pool.write_rows(batch.seq_pages[r.seq_id], k, v)
    ft = HH.DeviceFtState(cfg, L, ia3=use_ia3)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages, args.kv_split_pages)
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

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def forward(ly, ftc, wsx):
        if use_ia3:
            B.flexco_layer_forward_ia3(ly.c, ly.w, ia3.c, db.maps, x, y, pool.c, ftc, wsx.ptr, wsx.bytes)
        else:
            B.flexco_layer_forward(ly.c, ly.w, ly.lora, db.maps, x, y, pool.c, ftc, wsx.ptr, wsx.bytes)

    def backward(ly, pages, ftc, wsx, stream=None):
        if use_ia3:
            B.flexco_ia3_bwd(ly.c, ly.w, ia3.c, pool.c, pages, n_ft_pages, ftc, ft_req.start_pos, ft_req.n_new, dY, dX,
                             wsx.ptr, wsx.bytes, stream=stream)
        else:
            B.flexco_lora_bwd(ly.c, ly.w, ly.lora, pool.c, pages, n_ft_pages, ftc, ft_req.start_pos, ft_req.n_new, dY, dX,
                              wsx.ptr, wsx.bytes, stream=stream)

    def step_serial(i):
        ly = layers[i % len(layers)]
        forward(ly, ft.c, ws)
        backward(ly, ft_pages, ft.c, ws)

    def make_overlap_step():
        # The backward window of an iteration belongs to a sequence whose forward passes ran in earlier
        # iterations (Alg. 2: all forward windows, then the backward windows).  That sequence gets pages
        # and finetune state of its own - copies of what one forward of the batch leaves behind - so the
        # two streams touch disjoint data, the frozen weights and LoRA factors (both only read) apart.
        forward(layers[0], ft.c, ws)
        torch.cuda.synchronize()
        src_pages = ft_pages.long()
        bwd_pages = torch.arange(batch.num_pages, batch.num_pages + n_ft_pages, device="cuda")
        pool.k[bwd_pages] = pool.k[src_pages]
        pool.v[bwd_pages] = pool.v[src_pages]
        ft_b = HH.DeviceFtState(cfg, L, ia3=use_ia3)
        for name in ("q_cache", "attn", "x", "x2", "gate", "up", "lse") + (("k0", "v0") if use_ia3 else ()):
            getattr(ft_b, name).copy_(getattr(ft, name))
        bwd_pages = bwd_pages.to(torch.int32)
        ws_b = HH.Workspace(layers[0].c, T, hm.n_parts, n_ft, L)
        side = torch.cuda.Stream()
        torch.cuda.synchronize()

        def step_two_streams(i):
            ly = layers[i % len(layers)]
            forward(ly, ft.c, ws)
            backward(ly, bwd_pages, ft_b.c, ws_b, stream=side)
        step_two_streams.keep = (ft_b, ws_b, bwd_pages, side)
        return step_two_streams

    step = make_overlap_step() if args.overlap else step_serial

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- which kernel class dominates?  a short pass with every class bracketed by events -------
    probe_steps = 3
    for name, kid in B.KERNEL_IDS.items():
        B.flexco_kernel_timer_start(kid, 64 * probe_steps)
    for i in range(probe_steps):
        step_serial(i)      # one stream: every class's launches run alone, durations are the kernels' own
    torch.cuda.synchronize()
    probe = {}
    for name, kid in B.KERNEL_IDS.items():
        ms, n = B.flexco_kernel_timer_stop(kid)
        probe[name] = (ms / probe_steps, n / probe_steps)
    # the dominant kernel = the class whose single launch takes longest (the forward projections are four
    # launches of different shapes that together take about as long as the one attention launch; picking
    # by the class total would flip between the two from run to run)
    dominant = max(probe, key=lambda k: probe[k][0] / max(1.0, probe[k][1]))
    log("per-step kernel classes (ms): " + ", ".join("%s=%.3f" % (k, v[0]) for k, v in probe.items()))

    # ---- the timed region: K steps, the dominant class bracketed by events ---------------------
    # (a timed launch keeps its neighbours on the stream apart by a few microseconds, so only every
    # stride-th launch of the class carries events: with stride = launches per step + 1 the samples
    # rotate through the step's launches and weigh them equally)
    dom_per_step = int(round(probe[dominant][1]))
    stride = dom_per_step + 1
    B.flexco_kernel_timer_sample(B.KERNEL_IDS[dominant], stride)
    B.flexco_kernel_timer_start(B.KERNEL_IDS[dominant], 64 * args.steps)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    marks = []                                     # one event per step end (one-stream mode): median / min per step
    for i in range(args.steps):
        step(i)
        if not args.overlap:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            marks.append(e)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    per_step = [a.elapsed_time(b) for a, b in zip([ev0] + marks[:-1], marks)]
    dom_ms, dom_timed = B.flexco_kernel_timer_stop(B.KERNEL_IDS[dominant])
    B.flexco_kernel_timer_sample(B.KERNEL_IDS[dominant], 1)
    # with two streams the events on the forward's stream do not bracket the backward: wall clock only
    ms_per_step = (wall_ms if args.overlap else max(wall_ms, gpu_ms)) / args.steps
    value = T / (ms_per_step * 1e-3)

    work = algorithmic_work(cfg, batch, hm, db.numpy())
    roofline = roofline_entry(dominant, dom_ms / max(1, dom_timed), float(dom_per_step), work)
    roofline["timed_launches"] = dom_timed
    # the projections are as large a share of the step as the dominant kernel: their class figures beside it
    for gk in ("gemm_fwd", "gemm_bwd"):
        if probe.get(gk, (0, 0))[1] > 0:
            ge = roofline_entry(gk, probe[gk][0] / probe[gk][1], probe[gk][1], work)
            roofline["also_" + gk] = {"bound": ge["bound"], "achieved": ge["achieved"], "peak": ge["peak"], "unit": ge["unit"],
                                      "frac": ge["frac"], "ms_per_step": round(probe[gk][0], 4)}
            if "weight_stream_frac_of_hbm" in ge:
                roofline["also_" + gk]["weight_stream_frac_of_hbm"] = ge["weight_stream_frac_of_hbm"]
    roofline["timing"] = "HIP events on every %d-th launch of the class inside the timed region" % stride
    classes = {}
    for name, (ms, n) in probe.items():
        if n > 0:
            e = roofline_entry(name, ms / n, n, work)
            classes[name] = {"ms_per_step": round(ms, 4), "launches_per_step": n, "achieved": e["achieved"],
                             "unit": e["unit"], "frac": e["frac"], "bound": e["bound"]}
            if "weight_stream_frac_of_hbm" in e:
                classes[name]["weight_stream_frac_of_hbm"] = e["weight_stream_frac_of_hbm"]
    out = {
        "metric": "co-served tokens/s per layer iteration",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c2_llama8b_layer: 1 LLaMA-3.1-8B-shaped layer, T=1024 = 256 decode (ctx U[512,4096], "
                               "page 16) + 2x256 prefill + 256 finetune (last window of 2048); forward of all "
                               "tokens + " + ("(IA)^3 (k, v, FFN activation) window backward" if use_ia3 else
                                              "LoRA r16 (q,k,v,o,down) window backward"),
                   "tokens": T, "finetune_tokens": n_ft, "requests": hm.n_req,
                   "cached_positions": int(sum(r.start_pos + r.n_new for r in batch.requests)),
                   "weight_copies_cycled": len(layers),
                   "streams": "forward and window backward concurrent on two streams" if args.overlap else "one stream"},
        "roofline": roofline,
        "kernel_classes": classes,
        "gpu_event_ms_per_step": gpu_ms / args.steps,
    }
    if per_step:
        out["ms_per_step_median"] = float(np.median(per_step))
        out["ms_per_step_min"] = float(np.min(per_step))
    out["forward_projections"] = per_projection(B, torch, step_serial, cfg, T)
    # bf16 launches that missed the matrix-core kernels and ran type-generic ones (all zero at this configuration)
    out["bf16_generic_fallbacks"] = {k: v for k, v in B.flexco_bf16_fallbacks().items() if k in ("gemm_fwd", "gemm_bwd", "attn_fwd", "attn_bwd")}
    out["measured_ceilings"] = measured_ceilings(B, torch)
    if not args.overlap and not args.no_two_stream:
        # the same K steps again with the window backward on a second stream (reported beside the
        # one-stream figures above, which stay the headline: their kernel durations are undisturbed)
        step2 = make_overlap_step()
        for i in range(args.warmup):
            step2(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step2(i)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) * 1e3 / args.steps
        out["two_streams"] = {"value": T / (ms2 * 1e-3), "unit": "tokens/s", "ms_per_step": ms2,
                              "what": "same steps, the window backward on a second stream concurrent with the "
                                      "forward (Sec. 6.2 of the paper), on a finetune sequence of its own"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, batch, sample, W, lora, seed, x_np, ft_req, L, ia3_np)
    print(json.dumps(out), flush=True)


def per_projection(B, torch, step_serial, cfg, T):
    """The four forward projections one by one (three extra steps with an event pair on every launch of the class;
    a projection whose tile plan is two launches is the sum of both)."""
    kid = B.KERNEL_IDS["gemm_fwd"]
    steps = 3
    B.flexco_kernel_timer_sample(kid, 1)
    B.flexco_kernel_timer_start(kid, 16 * steps)
    for i in range(steps):
        step_serial(i)
    torch.cuda.synchronize()
    each = B.flexco_kernel_timer_read(kid)
    _, calls = B.flexco_kernel_timer_stop(kid)
    per_step = len(each) // steps
    H, F, qd, kd = cfg.hidden, cfg.ffn, cfg.q_dim, cfg.kv_dim
    names = [("qkv", (qd + 2 * kd) * H), ("o", qd * H), ("gate_up", 2 * F * H), ("down", F * H)]
    if calls != 4 * steps or per_step < 4 or len(each) != per_step * steps:
        return {"note": "unexpected launch pattern: %d pairs for %d calls" % (len(each), calls)}
    # the calls come in the order qkv, o, gate/up, down; extra pairs of a step belong to the widest projection
    # (gate/up), whose plan is the one that splits into two launches at this size
    extra = per_step - 4
    out = {}
    for k, (name, p) in enumerate(names):
        lo = k if k < 2 else (2 if k == 2 else 3 + extra)
        hi = lo + (1 + extra if k == 2 else 1)
        ms = sum(sum(each[st * per_step + j] for j in range(lo, hi)) for st in range(steps)) / steps
        tf = 2.0 * p * T / (ms * 1e-3) / 1e12
        out[name] = {"ms": round(ms, 4), "launches": hi - lo, "achieved": tf, "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS}
    return out


def measured_ceilings(B, torch):
    """What this GPU sustains for the two roofline resources, with the library's probe kernels: an MFMA
    loop on register operands and a contiguous read stream (each timed with events, best of 3)."""
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    buf = torch.empty(4 << 30, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best_mfma, best_read = 0.0, 0.0
    for rep in range(4):
        ev0.record()
        flops = B.flexco_probe_mfma(256, 20000, sink)
        ev1.record()
        torch.cuda.synchronize()
        if rep:
            best_mfma = max(best_mfma, flops / (ev0.elapsed_time(ev1) * 1e-3) / 1e12)
        ev0.record()
        nbytes = B.flexco_probe_read(buf, buf.numel(), 2048, sink)
        ev1.record()
        torch.cuda.synchronize()
        if rep:
            best_read = max(best_read, nbytes / (ev0.elapsed_time(ev1) * 1e-3) / 1e9)
    # the matrix cores fed from LDS as the projection kernels feed them: without and with the stage's tile loads
    # (from a cache-resident 512 KB) and barrier
    best_lds = {}
    for tile in (128, 256):
        for loads in (False, True):
            best = 0.0
            for rep in range(3):
                ev0.record()
                flops = B.flexco_probe_mfma_lds(256, 4000 if tile == 128 else 1000, tile, sink, buf if loads else None,
                                                1 << 20 if loads else 0)
                ev1.record()
                torch.cuda.synchronize()
                if rep:
                    best = max(best, flops / (ev0.elapsed_time(ev1) * 1e-3) / 1e12)
            best_lds[(tile, loads)] = best
    # plain device-to-device copy of 1 GiB (read + write counted)
    src, dst = buf[:1 << 30], buf[1 << 30:2 << 30]
    best_copy = 0.0
    for rep in range(4):
        ev0.record()
        dst.copy_(src)
        ev1.record()
        torch.cuda.synchronize()
        if rep:
            best_copy = max(best_copy, 2.0 * (1 << 30) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9)
    del src, dst, buf
    return {"mfma_bf16_loop_tflops": best_mfma,
            "mfma_bf16_lds_operands_tile128_tflops": best_lds[(128, False)],
            "mfma_bf16_lds_operands_tile256_tflops": best_lds[(256, False)],
            "k_loop_without_memory_wait_tile128_tflops": best_lds[(128, True)],
            "k_loop_without_memory_wait_tile256_tflops": best_lds[(256, True)], "hbm_read_stream_gbs": best_read,
            "device_copy_gbs": best_copy,
            "what": "probe kernels of the library: 256 blocks x 4 wavefronts of back-to-back v_mfma_f32_32x32x16_bf16 on "
                    "register operands in [-1, 1); the same products with operands read from LDS in the projection "
                    "kernels' pattern for a 128 x 128 and a 256 x 256 block tile, one slice ahead (no global traffic, no "
                    "barriers), and with a stage of tile loads into LDS from cache-resident memory plus a barrier per "
                    "stage (the kernels' k-loop minus its wait for memory); "
                    "2048 blocks streaming 4 GiB with 16-byte loads; a 1 GiB device-to-device "
                    "copy (bytes read + bytes written)"}


def algorithmic_work(cfg, batch, hm, maps_np=None):
    """Algorithmic flops / bytes per STEP of each kernel class: what the method must move or multiply, in the
    storage type (2 bytes; 4 for the fp32 accumulators and log-sum-exp), each operand of each operator read or
    written once - not what this implementation's split-K partial sums or by-products add."""
    H, F, r = cfg.hidden, cfg.ffn, cfg.lora_rank
    qd, kd, nq = cfg.q_dim, cfg.kv_dim, cfg.n_q_heads
    T, n = hm.T, hm.n_ft
    e = 2
    p_base = (qd + 2 * kd) * H + qd * H + 3 * H * F
    # attention forward: every cached position a request sees is read once, K row + V row of every kv head
    kv_bytes = sum((q.start_pos + q.n_new) * 2 * kd * e for q in batch.requests)
    ftr = [q for q in batch.requests if q.kind == 2]
    bwd_flops = 0.0
    for q in ftr:
        s_, l = q.n_new, q.start_pos + q.n_new
        vis = s_ * (l - s_) + s_ * (s_ + 1) / 2
        bwd_flops += 10.0 * nq * cfg.head_dim * vis
    # row-wise operators (norms, rotation + cache append, SwiGLU backward, rotation backward, norm backwards)
    fwd_rows = (2 * T * H + n * H) * e                      # norm 1: x in, h out, the window's x rows kept
    fwd_rows += (2 * T * (qd + 2 * kd) + n * qd) * e        # rotation: q, k, v in; q, K / V pages out; Q cache rows
    fwd_rows += (2 * T * H + n * H) * e                     # norm 2: x2 in, h2 out, the window's x2 rows kept
    bwd_rows = (3 * n * F + 2 * n * F + n * F) * e          # SwiGLU backward: gate, up, d(act) in; d(gate), d(up), act out
    bwd_rows += (3 * n * H + 2 * n * H) * e                 # norm 2 backward: x2, d(h2), dY in; d(x2), h2 out
    bwd_rows += n * qd * e + 2 * n * kd * 4 + n * (qd + 2 * kd) * e     # rotation backward: dQ, the accumulators' rows in; dq, dk, dv out
    bwd_rows += (3 * n * H + 2 * n * H) * e                 # norm 1 backward: x, d(h1), d(x2) in; dX, h1 out
    # the bypass networks: every target reads its input rows and (backward) its output-gradient rows twice
    # (rank-r product, then the two weight-gradient products), plus the r-wide matrices
    dims = {"q": (H, qd), "k": (H, kd), "v": (H, kd), "o": (qd, H), "gate": (H, F), "up": (H, F), "down": (F, H)}
    lora_b = 0.0
    for t in cfg.lora_targets:
        i_, o_ = dims[t]
        lora_b += (hm.n_lora * i_ + r * i_) * e                            # forward: x rows and A
        lora_b += (2 * n * i_ + 2 * n * o_ + 2 * r * (i_ + o_)) * e         # backward: x, dy rows (twice), A, B
        lora_b += 2 * r * (i_ + o_) * 4                                     # dA, dB read-modify-write (fp32)
    # split merge: the partial rows of the tiles whose key range was cut, the output rows and log-sum-exp
    merge_b = (T * qd * e + T * nq * 4)
    if maps_np is not None:
        cut = maps_np["tile_nsplit"][maps_np["tile_nsplit"] > 1]
        group = nq // cfg.n_kv_heads
        cols = max(1, 16 // group) * group
        merge_b += float(cut.sum()) * cfg.n_kv_heads * cols * (cfg.head_dim + 2) * 4
    return {
        "gemm_fwd": ("mfma", 2.0 * p_base * T),
        "gemm_bwd": ("mfma", 2.0 * p_base * n),
        "attn_fwd": ("hbm", float(kv_bytes)),
        "attn_bwd": ("mfma", bwd_flops),
        "elemwise": ("hbm", float(fwd_rows + bwd_rows)),
        "lora": ("hbm", float(lora_b)),
        "attn_merge": ("hbm", float(merge_b)),
        "weights_bytes": 2.0 * p_base,
    }


def measured_traffic(kernel_class):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "traffic_%s_c2.txt" % kernel_class)
    if not os.path.exists(path):
        return None
    m = re.search(r"hbm_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read())
    return float(m.group(1)) if m else None


def roofline_entry(name, avg_launch_ms, launches_per_step, work):
    kind, per_step = work.get(name, ("hbm", None))
    base = {"kernel": KERNEL_NAMES.get(name, name), "class": name, "avg_launch_ms": avg_launch_ms,
            "launches_per_step": launches_per_step, "traffic": measured_traffic(name)}
    if per_step is None or launches_per_step == 0:
        base.update({"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None})
        return base
    per_launch = per_step / launches_per_step
    if kind == "mfma":
        ach = per_launch / (avg_launch_ms * 1e-3) / 1e12
        base.update({"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops_per_launch": per_launch})
        if name == "gemm_bwd":   # below the ridge the weight stream bounds it: report that too
            gbs = work["weights_bytes"] / launches_per_step / (avg_launch_ms * 1e-3) / 1e9
            base["weight_stream_GBs"] = gbs
            base["weight_stream_frac_of_hbm"] = gbs / HBM_PEAK_GBS
    else:
        ach = per_launch / (avg_launch_ms * 1e-3) / 1e9
        base.update({"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": per_launch})
    return base


def cpu_baseline(cfg, batch, sample, W, lora, seed, x_np, ft_req, L, ia3=None):
    """The oracle, as it stands, on a bounded sample of the same workload (forward of the sampled
    requests' tokens + the finetune window's backward), timed on this machine's host cores."""
    from oracle import layer as OL
    from oracle import ia3 as OI
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
    st = {ft_req.seq_id: OI.Ia3FtState(cfg, L) if ia3 is not None else OL.FtState(cfg, L)}
    threads = sum(p.get("num_threads", 0) for p in threadpoolctl.threadpool_info() if p.get("user_api") == "blas") or os.cpu_count()
    log("cpu baseline: oracle on %d sampled tokens (%d requests), %d BLAS threads" % (len(rows), len(sample), threads))
    dY = gen.layer_input(cfg, seed, ft_req.n_new, tag="dy")
    sl = pool.slots(batch.seq_pages[ft_req.seq_id], L)
    # repeat the sample until about 10 s of oracle time have been spent (at most 6 passes)
    t_f = t_b = 0.0
    reps = 0
    while reps < 6 and (t_f + t_b) < 10.0:
        t0 = time.perf_counter()
        if ia3 is not None:
            OI.forward_mixed(cfg, W, ia3, om, x_np[rows], pool, st)
        else:
            OL.layer_forward_mixed(cfg, W, lora, om, x_np[rows], pool, st)
        t_f += time.perf_counter() - t0
        t0 = time.perf_counter()
        kk, vv = pool.k[sl].astype(np.float64), pool.v[sl].astype(np.float64)
        if ia3 is not None:
            OI.backward_window(cfg, W, ia3, st[ft_req.seq_id], kk, vv, ft_req.start_pos, ft_req.n_new, dY, {})
        else:
            OL.layer_backward_window(cfg, W, lora, st[ft_req.seq_id], kk, vv, ft_req.start_pos, ft_req.n_new, dY, {})
        t_b += time.perf_counter() - t0
        reps += 1
    log("cpu baseline: %d passes, forward %.1fs, backward %.1fs, total incl. setup %.1fs" % (reps, t_f, t_b, time.time() - t_all))
    return {"value": reps * len(rows) / (t_f + t_b), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d of 1024 tokens (%d decode requests, the two 256-token prefill chunks, the 256-token finetune "
                      "window): forward + that window's backward, %d passes; numpy fp64" % (len(rows), len(sample) - 3, reps),
            "seconds": t_f + t_b, "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
