"""Times the two attention entry points on their own, on the batches of a configuration:

    python -m paper_2402_18789_amd.attn_bench [--config c2|c3|c4|c5] [--inference-share S] [--reps 10]

* flexco_attention_mixed (Sec. 6.2: decode tokens, prefill chunks and finetune windows in one call) on the
  configuration's mixed batch, on its decode requests alone, on its chunk requests alone (prefill + finetune
  window: a decode-free iteration), under every setting of flexco_attention_chunk_path: 0 = one kernel for
  everything, 1 = the chunk items on the four-wavefront kernel after the decode tokens' kernel, 2 = beside it on
  the library's side stream, -1 = the library's own choice by batch;
* flexco_attention_window_bwd (Alg. 2, the window's dQ and the accumulated dK / dV) on the configuration's
  finetune window.

Synthetic caches and queries (the timing does not depend on the values); prints one line per case.  FLOP
figures count 4 d per (row, visible key, head) forward and 10 d backward (the five products of the definition).
"""
import argparse

import torch

import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH
from workload import gen
from workload.configs import CONFIGS, KIND_DECODE, KIND_FINETUNE

BATCHES = {
    "c2": ("c2_llama8b_layer", gen.batch_c2),
    "c3": ("c3_llama8b_full", gen.batch_c3),
    "c4": ("c4_qwen14b_full", gen.batch_c4),
    "c5": ("c5_qwen32b_full", gen.batch_c5),
}
MODES = ((0, "one kernel"), (1, "chunk kernel after"), (2, "chunk kernel beside"), (-1, "default"))


def time_us(fn, reps):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(3):
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps * 1e3)
    return best


def forward_cases(cfg, batch, reps):
    pools = [HH.DevicePool(cfg, batch.num_pages) for _ in range(2)]     # two copies in turn: nothing stays cached
    for i, p in enumerate(pools):
        p.fill_random(i)
    dcfg = HH.c_cfg(cfg)
    dec = [r for r in batch.requests if r.kind == KIND_DECODE]
    oth = [r for r in batch.requests if r.kind != KIND_DECODE]
    for name, reqs in (("mixed batch", batch.requests), ("decode requests", dec), ("chunk requests", oth)):
        if not reqs:
            continue
        db = HH.DeviceBatch(cfg, reqs, batch.seq_pages, batch.num_pages)
        hm = db.host_maps
        ws = HH.Workspace(dcfg, hm.T, hm.n_parts)
        q = torch.randn(hm.T, cfg.q_dim, device="cuda").bfloat16()
        out = torch.empty_like(q)
        lse = torch.empty((hm.T, cfg.n_q_heads), dtype=torch.float32, device="cuda")
        turn = [0]

        def call():
            turn[0] ^= 1
            B.flexco_attention_mixed(dcfg, db.maps, q, pools[turn[0]].c, out, lse, ws.ptr, ws.bytes)

        us = {}
        try:
            for mode, _ in MODES:
                B.flexco_attention_chunk_path(mode)
                us[mode] = time_us(call, reps)
        finally:
            B.flexco_attention_chunk_path(-1)
        vis_dec = sum(r.start_pos + r.n_new for r in reqs if r.kind == KIND_DECODE)
        vis_chunk = sum(r.n_new * r.start_pos + r.n_new * (r.n_new + 1) // 2 for r in reqs if r.kind != KIND_DECODE)
        kv_bytes = vis_dec * cfg.n_kv_heads * cfg.head_dim * 2 * 2
        flops = 4.0 * cfg.n_q_heads * cfg.head_dim * (vis_dec + vis_chunk)
        line = "forward  %-16s T=%5d items=%5d (one-token %5d) split=%3d pages  stream %6d pages, chunks %6d tile-pages:" % (
            name, hm.T, hm.n_items, hm.n_single, hm.kv_split_pages, hm.stream_pages, hm.chunk_tile_pages)
        line += "".join("  %s %.1f us" % (label, us[mode]) for mode, label in MODES)
        d = us[-1]
        line += "   (default: %.2f TB/s of decode K/V, %.0f TFLOP/s)" % (kv_bytes / d / 1e6, flops / d / 1e6)
        print(line, flush=True)


def backward_case(cfg, batch, reps):
    ft = [r for r in batch.requests if r.kind == KIND_FINETUNE]
    if not ft:
        return
    s, l = ft[0].n_new, ft[0].start_pos + ft[0].n_new
    n_pages = (l + cfg.page_size - 1) // cfg.page_size
    pool = HH.DevicePool(cfg, n_pages + 2)
    pool.fill_random(1)
    pages = torch.arange(1, n_pages + 1, dtype=torch.int32, device="cuda")
    q = torch.randn(s, cfg.q_dim, device="cuda").bfloat16()
    o = torch.randn(s, cfg.q_dim, device="cuda").bfloat16() * 0.1
    do = torch.randn(s, cfg.q_dim, device="cuda").bfloat16()
    lse = torch.full((s, cfg.n_q_heads), 40.0, device="cuda")
    dq = torch.empty_like(q)
    dk = torch.zeros(l, cfg.kv_dim, device="cuda")
    dv = torch.zeros_like(dk)
    ws = torch.empty(s * cfg.n_q_heads * 4 + 1024, dtype=torch.uint8, device="cuda")
    dcfg = HH.c_cfg(cfg)
    us = time_us(lambda: B.flexco_attention_window_bwd(dcfg, pool.c, pages, n_pages, l - s, s, q, o, lse, do, dq, dk, dv,
                                                       ws, ws.numel()), reps)
    vis = s * (l - s) + s * (s + 1) / 2
    flops = 10.0 * cfg.n_q_heads * cfg.head_dim * vis
    print("backward window of %d rows on a prefix of %d, %d query heads per kv head: %.1f us  %.0f TFLOP/s" % (
        s, l - s, cfg.n_q_heads // cfg.n_kv_heads, us, flops / us / 1e6), flush=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", choices=sorted(BATCHES), default="c2")
    ap.add_argument("--inference-share", type=float, default=None, help="c4 only: share of the token budget that is inference")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("attn_bench needs the GPU")
    name, make = BATCHES[args.config]
    cfg = CONFIGS[name]
    if args.inference_share is not None:
        if args.config != "c4":
            raise SystemExit("--inference-share goes with --config c4")
        batch = make(args.seed, args.inference_share)
    else:
        batch = make(args.seed)
    print("%s%s" % (name, "" if args.inference_share is None else ", inference share %g" % args.inference_share), flush=True)
    forward_cases(cfg, batch, args.reps)
    backward_case(cfg, batch, args.reps)


if __name__ == "__main__":
    main()
