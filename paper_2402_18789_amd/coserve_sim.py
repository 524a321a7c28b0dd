"""Co-serving with the hybrid token scheduler (Sec. 6.2) on one GPU.

1. Profiles the latency functions the scheduler needs from this library's own kernels, on the 8B
   layer shape: f_fwd(c, s) = one layer's forward over c inference tokens + a finetuning window of
   s tokens (one fused batch); f_bwd(c, s) = that layer's forward over c inference tokens with the
   backward of an s-token window running on a second stream (Sec. 6.2 runs the backward pass of
   finetuning tokens on its own stream).  An iteration of the n-layer model is taken as n_layers times
   the per-layer figure.
2. Checks the interpolated model against fresh measurements at points off the grid.
3. Runs the two-stage scheduler (library calls) over a seeded synthetic arrival process in virtual
   time - each iteration advances the clock by the model's estimate - and reports, per arrival rate,
   inference tokens/s, finetuned tokens/s and the latency of the iterations against the SLO.

The request lengths stand in for the traces the paper uses (not available offline): prompt and
generation lengths are seeded log-normal draws.  Run on an MI355X:
    python -m paper_2402_18789_amd.coserve_sim [--out FILE]
"""
import argparse
import sys
import time

import numpy as np
import torch

from workload import gen, CONFIGS
from . import binding as B
from . import host as HH

C_GRID = [32, 128, 256, 512, 768, 1024]
S_GRID = [0, 64, 128, 256, 512]
FT_LEN = 2048              # tokens of a finetuning sequence
N_LAYERS = 32


def mix(c):
    """c inference tokens as the benchmark mixes them: a third decode tokens (at most 256), the rest
    prompt chunks of at most 256 tokens."""
    n_dec = min(256, c // 3)
    rest = c - n_dec
    chunks = [256] * (rest // 256) + ([rest % 256] if rest % 256 else [])
    return n_dec, chunks


class Bed:
    """Device state for timing one layer on arbitrary (c, s) batches."""

    def __init__(self, seed=0):
        self.cfg = CONFIGS["c2_llama8b_layer"]
        self.seed = seed
        cfg = self.cfg
        self.layer = HH.DeviceLayer(cfg, gen.layer_weights(cfg, seed, 0), gen.lora_weights(cfg, seed, 0))
        self.side = torch.cuda.Stream()
        self.cache = {}

    def batch(self, c, s):
        key = (c, s)
        if key in self.cache:
            return self.cache[key]
        cfg = self.cfg
        n_dec, chunks = mix(c)
        ctx = gen.rng(self.seed, "coserve", "ctx", c).integers(512, 4097, size=n_dec)
        prefill = [(0, n, n) for n in chunks]
        finetune = [(FT_LEN - s, s, FT_LEN)] if s else []
        # the backward's own sequence: always present, so that f_bwd can use it (no tokens in the batch
        # when s = 0: it is appended as a second finetune-length sequence's pages only)
        b = gen.mixed_batch(cfg.page_size, self.seed, decode_ctx=ctx, prefill=prefill, finetune=finetune)
        extra = -(-FT_LEN // cfg.page_size)
        pool = HH.DevicePool(cfg, b.num_pages + extra)
        pool.fill_random(self.seed)
        db = HH.DeviceBatch(cfg, b.requests, b.seq_pages, b.num_pages + extra)
        T = db.host_maps.T
        ft = HH.DeviceFtState(cfg, FT_LEN)
        ft_b = HH.DeviceFtState(cfg, FT_LEN)
        g = torch.Generator(device="cuda")
        g.manual_seed(self.seed + 1)
        for name in ("q_cache", "attn", "x", "x2", "gate", "up"):
            t = getattr(ft_b, name)
            t.copy_(torch.randn(t.shape, generator=g, device="cuda", dtype=torch.float32).to(t.dtype))
        ft_b.lse.fill_(8.0)
        ws = HH.Workspace(self.layer.c, max(T, 1), db.host_maps.n_parts, 512, FT_LEN)
        ws_b = HH.Workspace(self.layer.c, 1, 1, 512, FT_LEN)
        x = torch.randn((T, cfg.hidden), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        y = torch.empty_like(x)
        dY = torch.randn((512, cfg.hidden), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        dX = torch.empty_like(dY)
        bwd_pages = torch.arange(b.num_pages, b.num_pages + extra, device="cuda", dtype=torch.int32)
        st = dict(db=db, pool=pool, ft=ft, ft_b=ft_b, ws=ws, ws_b=ws_b, x=x, y=y, dY=dY, dX=dX, bwd_pages=bwd_pages,
                  n_bwd_pages=extra, has_ft=bool(s))
        if len(self.cache) > 4:
            self.cache.clear()
        self.cache[key] = st
        return st

    def forward(self, st):
        ly = self.layer
        B.flexco_layer_forward(ly.c, ly.w, ly.lora, st["db"].maps, st["x"], st["y"], st["pool"].c,
                               st["ft"].c if st["has_ft"] else None, st["ws"].ptr, st["ws"].bytes)

    def backward(self, st, s):
        ly = self.layer
        B.flexco_lora_bwd(ly.c, ly.w, ly.lora, st["pool"].c, st["bwd_pages"], st["n_bwd_pages"], st["ft_b"].c,
                          FT_LEN - s, s, st["dY"][:s], st["dX"][:s], st["ws_b"].ptr, st["ws_b"].bytes, stream=self.side)

    def time_fwd(self, c, s, reps=5):
        st = self.batch(c, s)
        return self._time(lambda: self.forward(st), reps)

    def time_bwd(self, c, s, reps=5):
        """forward over the c inference tokens with the backward of an s-token window on the side stream"""
        st = self.batch(c, 0)
        if s == 0:
            return self._time(lambda: self.forward(st), reps)

        def both():
            self.forward(st)
            self.backward(st, s)
        return self._time(both, reps)

    @staticmethod
    def _time(fn, reps):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        best = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            best.append((time.perf_counter() - t0) * 1e3)
        return float(np.median(best))


def profile(bed, log):
    fwd = np.zeros((len(C_GRID), len(S_GRID)), np.float32)
    bwd = np.zeros_like(fwd)
    for i, c in enumerate(C_GRID):
        for j, s in enumerate(S_GRID):
            fwd[i, j] = bed.time_fwd(c, s)
            bwd[i, j] = bed.time_bwd(c, s)
        log("profiled c=%4d: fwd %s | with backward %s" % (c, " ".join("%.3f" % v for v in fwd[i]),
                                                          " ".join("%.3f" % v for v in bwd[i])))
    return fwd, bwd


def simulate(model_f, model_b, rate, slo_ms, horizon_s, seed, max_batch=256, token_budget=768, chunk=256, quantum=16):
    """Virtual-time run of the two-stage scheduler.  Returns a dict of totals."""
    g = gen.rng(seed, "coserve", "arrivals", rate)
    n = int(rate * horizon_s * 1.5) + 16
    arrive = np.cumsum(g.exponential(1.0 / rate, n))
    prompt_all = np.clip(np.exp(g.normal(np.log(256.0), 0.8, n)), 16, 2048).astype(np.int32)
    gen_all = np.clip(np.exp(g.normal(np.log(128.0), 0.8, n)), 1, 512).astype(np.int32)
    cap = n
    prompt, gen_len = np.ones(cap, np.int32), np.zeros(cap, np.int32)
    prefilled, generated = np.zeros(cap, np.int32), np.zeros(cap, np.int32)
    state = np.full(cap, B.FLEXCO_REQ_FINISHED, np.int32)
    prefilled[:] = 1                                   # unused slots: a finished one-token request
    now, nxt = 0.0, 0
    ft_fwd, ft_bwd, ft_done = 0, 0, 0                  # cursor of the current sequence, sequences finished
    out = dict(iters=0, inf_tokens=0, gen_tokens=0, ft_fwd_tokens=0, ft_bwd_tokens=0, lat=[], over=0)
    layers_slo = slo_ms / N_LAYERS
    while now < horizon_s:
        while nxt < n and arrive[nxt] <= now:          # admit arrivals into the request table
            prompt[nxt], gen_len[nxt] = prompt_all[nxt], gen_all[nxt]
            prefilled[nxt], generated[nxt], state[nxt] = 0, 0, B.FLEXCO_REQ_WAITING
            nxt += 1
        live = slice(0, max(nxt, 1))
        entries, c = B.flexco_sched_inference(prompt[live], prefilled[live], gen_len[live], generated[live], state[live],
                                              max_batch, token_budget, chunk)
        # stage 2: forward windows until the sequence is covered, then backward windows from its end
        if ft_fwd < FT_LEN:
            s = B.flexco_sched_window(model_f, c, layers_slo, min(512, FT_LEN - ft_fwd), quantum)
            lat = B.flexco_latency_estimate(model_f, c, s)
            ft_fwd += s
            out["ft_fwd_tokens"] += s
        else:
            s = B.flexco_sched_window(model_b, c, layers_slo, min(512, FT_LEN - ft_bwd), quantum)
            lat = B.flexco_latency_estimate(model_b, c, s)
            ft_bwd += s
            out["ft_bwd_tokens"] += s
            if ft_bwd >= FT_LEN:
                ft_fwd, ft_bwd, ft_done = 0, 0, ft_done + 1
        if c == 0 and s == 0:                          # idle: jump to the next arrival
            now = arrive[nxt] if nxt < n else horizon_s
            continue
        B.flexco_sched_advance(entries, prompt[live], prefilled[live], gen_len[live], generated[live], state[live])
        lat_ms = lat * N_LAYERS
        now += lat_ms * 1e-3
        out["iters"] += 1
        out["inf_tokens"] += c
        out["gen_tokens"] += int(sum(1 for e in entries if e[1] == B.FLEXCO_DECODE))
        out["lat"].append(lat_ms)
        out["over"] += lat_ms > slo_ms * (1 + 1e-9)
    out["time_s"], out["ft_sequences"] = now, ft_done
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=None)
    ap.add_argument("--slo-ms", type=float, default=50.0, help="per-iteration latency bound (time per output token)")
    ap.add_argument("--horizon-s", type=float, default=60.0)
    ap.add_argument("--rates", default="2,5,10,20,40")
    args = ap.parse_args(argv)
    lines = []

    def log(msg):
        print(msg, flush=True)
        lines.append(msg)

    assert torch.cuda.is_available(), "coserve_sim needs a GPU"
    bed = Bed()
    log("co-serving on the 8B layer shape, %d layers assumed per iteration, SLO %.0f ms per iteration" % (N_LAYERS, args.slo_ms))
    log("c grid %s, s grid %s; per-layer latencies in ms" % (C_GRID, S_GRID))
    fwd, bwd = profile(bed, log)
    model_f = B.HostLatencyModel(C_GRID, S_GRID, fwd)
    model_b = B.HostLatencyModel(C_GRID, S_GRID, bwd)
    # ---- the model against fresh measurements off the grid -------------------------------------
    errs = []
    for (c, s) in [(96, 32), (384, 192), (640, 96), (900, 384), (200, 448), (1000, 16)]:
        m = bed.time_fwd(c, s)
        e = B.flexco_latency_estimate(model_f, c, s)
        errs.append(abs(e - m) / m)
        log("check f_fwd(%4d, %3d): measured %.3f ms, model %.3f ms (%+.1f %%)" % (c, s, m, e, 100 * (e - m) / m))
    log("model vs measurement off the grid: mean |error| %.1f %%, max %.1f %%" % (100 * np.mean(errs), 100 * np.max(errs)))
    # ---- the scheduler over arrival rates -------------------------------------------------------
    log("")
    log("%8s %10s %12s %12s %14s %10s %10s %8s" % ("req/s", "iters", "inf tok/s", "gen tok/s", "finetune tok/s", "p50 ms", "p99 ms", "> SLO"))
    for rate in [float(r) for r in args.rates.split(",")]:
        r = simulate(model_f, model_b, rate, args.slo_ms, args.horizon_s, seed=0)
        lat = np.array(r["lat"]) if r["lat"] else np.zeros(1)
        # a token is finetuned once its forward and its backward window have both run
        ft_tok_s = min(r["ft_fwd_tokens"], r["ft_bwd_tokens"] + 0) / r["time_s"] if r["time_s"] else 0.0
        trained = (r["ft_sequences"] * FT_LEN + 0.0) / r["time_s"]
        log("%8.1f %10d %12.0f %12.0f %14.0f %10.1f %10.1f %8d" % (rate, r["iters"], r["inf_tokens"] / r["time_s"],
                                                                  r["gen_tokens"] / r["time_s"], trained, np.median(lat),
                                                                  np.percentile(lat, 99), r["over"]))
        del ft_tok_s
    log("")
    log("finetune tok/s = tokens of finetuning sequences whose forward and backward passes both completed, per second")
    if args.out:
        with open(args.out, "w") as f:
            f.write("\n".join(lines) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
