"""The whole-model iteration driver (forward through every layer, loss head, backward through every
layer, Adam) runs and leaves finite results; the numbers of the same calls chained over layers are
checked against the oracle in test_gpu_train.py and test_gpu_parity.py."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_model_iteration_two_layers():
    from paper_2402_18789_amd import model_iter
    say("model iteration, 2 layers of the 8B shape, vocabulary 4096")
    r = model_iter.run(n_layers=2, steps=1, warmup=1, vocab=4096)
    say(str({k: r[k] for k in ("ms_per_iteration", "forward_ms", "loss_head_ms", "backward_ms", "loss", "lora_grad_norm_dB")}))
    assert r["finite"]
    assert r["config"]["tokens"] == 2048 and r["config"]["finetune_tokens"] == 512
    # a random head's loss over the window's rows, scaled by window / sequence: ln(V) / 4 to a few percent
    import math
    assert abs(r["loss"] - math.log(4096) * 512 / 2048) < 0.2 * math.log(4096) * 512 / 2048
    assert r["lora_grad_norm_dB"] > 0
    assert r["forward_ms"] > 0 and r["backward_ms"] > 0


# ------------------------------------------------------------------------------------------------------------
# Three layers of the 8B shape chained, whole-model batch, against the oracle's own chain (no device value ever
# reaches the oracle): the device runs the full T = 2048 batch through three layers with weights, pools and
# finetune state of their own and the window's backward from a seeded top gradient back down; the oracle runs a
# sample of the requests (decode tokens, a whole prompt, the last truncated prompt, the finetune window) through
# the same three layers from the same seeded inputs.
# ------------------------------------------------------------------------------------------------------------
def _compact_pages(batch, sample):
    """the sampled sequences' page lists renumbered 0, 1, 2, ... for a small oracle-side pool (the oracle's results
    do not depend on which pages hold a sequence)"""
    import numpy as np
    out, nxt = {}, 0
    for r in sample:
        n = len(batch.seq_pages[r.seq_id])
        out[r.seq_id] = np.arange(nxt, nxt + n)
        nxt += n
    return out, nxt


def test_chain_of_three_layers_8b_shape_sampled():
    import numpy as np
    import torch
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from oracle import layer as OL
    from oracle.maps import build_maps
    from workload import gen, CONFIGS
    from gpu_common import assert_close_storage, to_np, TOL
    say("chain of three 8B-shaped layers on the whole-model batch, sampled")
    cfg, seed, N = CONFIGS["c3_llama8b_full"], 0, 3
    tol = TOL["bf16"]
    batch = gen.batch_c3(seed)
    sample = gen.sample_requests(batch, 8)
    ft_req = [r for r in batch.requests if r.kind == 2][0]
    L = batch.seq_capacity[ft_req.seq_id]
    Ws = [gen.layer_weights(cfg, seed, n) for n in range(N)]
    los = [gen.lora_weights(cfg, seed, n) for n in range(N)]
    devs = [HH.DeviceLayer(cfg, Ws[n], los[n]) for n in range(N)]
    pools = [HH.DevicePool(cfg, batch.num_pages) for _ in range(N)]
    fts = [HH.DeviceFtState(cfg, L) for _ in range(N)]
    cpages, n_cp = _compact_pages(batch, sample)
    o_pools = [OL.KVPool(n_cp, cfg.page_size, cfg.kv_dim, dtype=np.float32) for _ in range(N)]
    o_fts = [OL.FtState(cfg, L) for _ in range(N)]
    for n in range(N):
        pools[n].fill_random(seed + n)
        for r in sample:
            if r.start_pos:
                k, v = gen.kv_prefix(cfg, seed, n, r.seq_id, r.start_pos)
                pools[n].write_rows(batch.seq_pages[r.seq_id], k, v)
                sl = o_pools[n].slots(cpages[r.seq_id], r.start_pos)
                o_pools[n].k[sl], o_pools[n].v[sl] = k, v
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    hm = db.host_maps
    ws = HH.Workspace(devs[0].c, hm.T, hm.n_parts, ft_req.n_new, L)
    x_np = gen.layer_input(cfg, seed, hm.T)
    cur = torch.from_numpy(x_np).to("cuda", torch.bfloat16)
    say("  device: forward through %d layers, T = %d" % (N, hm.T))
    for n in range(N):
        out = torch.empty_like(cur)
        B.flexco_layer_forward(devs[n].c, devs[n].w, devs[n].lora, db.maps, cur, out, pools[n].c, fts[n].c, ws.ptr, ws.bytes)
        cur = out
    torch.cuda.synchronize()
    assert bool(torch.isfinite(cur.float()).all())
    dY_np = gen.layer_input(cfg, seed, ft_req.n_new, tag="dy_top")
    d_cur = torch.from_numpy(dY_np).to("cuda", torch.bfloat16)
    pages_d = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")
    for n in range(N - 1, -1, -1):
        d_next = torch.empty_like(d_cur)
        B.flexco_lora_bwd(devs[n].c, devs[n].w, devs[n].lora, pools[n].c, pages_d, int(pages_d.numel()), fts[n].c,
                          ft_req.start_pos, ft_req.n_new, d_cur, d_next, ws.ptr, ws.bytes)
        d_cur = d_next
    torch.cuda.synchronize()
    # ---- oracle: the sampled requests through the same chain, its own values all the way; once plain (the bar)
    # and once with every stored tensor rounded to bf16 (what the storage type alone costs, for the rule of
    # gpu_common.assert_close_storage) ----
    rows = gen.sample_token_rows(batch, sample)
    om = build_maps(sample, cpages, batch.page_size, n_cp)
    say("  oracle: %d sampled tokens through %d layers, plain and with bf16 storage" % (len(rows), N))
    res = {}
    for storage in (None, "bf16"):
        if storage is not None:                      # fresh caches and state for the second run
            for n in range(N):
                o_fts[n] = OL.FtState(cfg, L)
        h = x_np[rows].astype(np.float64)
        for n in range(N):
            h = OL.layer_forward_mixed(cfg, Ws[n], los[n], om, h, o_pools[n], {ft_req.seq_id: o_fts[n]}, storage=storage)
        out = {"top output (sampled rows)": h}
        sl = o_pools[0].slots(cpages[ft_req.seq_id], L)
        d = dY_np.astype(np.float64)
        grads = [dict() for _ in range(N)]
        for n in range(N - 1, -1, -1):
            d = OL.layer_backward_window(cfg, Ws[n], los[n], o_fts[n], o_pools[n].k[sl].astype(np.float64),
                                         o_pools[n].v[sl].astype(np.float64), ft_req.start_pos, ft_req.n_new, d, grads[n],
                                         storage=storage)
        out["dX below the bottom layer"] = d
        for n in range(N):
            out[f"layer {n} dk_accum"], out[f"layer {n} dv_accum"] = o_fts[n].dk_accum.copy(), o_fts[n].dv_accum.copy()
            for t in cfg.lora_targets:
                out[f"layer {n} dA[{t}]"], out[f"layer {n} dB[{t}]"] = grads[n][t]
        res[storage] = out
    got = {"top output (sampled rows)": to_np(cur)[rows], "dX below the bottom layer": to_np(d_cur)}
    for n in range(N):
        gg = devs[n].grads_numpy()
        got[f"layer {n} dk_accum"], got[f"layer {n} dv_accum"] = to_np(fts[n].dk_accum), to_np(fts[n].dv_accum)
        for t in cfg.lora_targets:
            got[f"layer {n} dA[{t}]"], got[f"layer {n} dB[{t}]"] = gg[t]
    report, excess, failures = [], [], []
    for name in res[None]:
        try:
            e, _ = assert_close_storage(name, got[name], res[None][name], res["bf16"][name], tol, report)
            if e > tol:
                excess.append(name)
        except AssertionError as err:
            failures.append(str(err))
    say("  device vs plain (bf16 storage alone vs plain): " + ", ".join(f"{r[0]}={r[1]:.1e}({r[2]:.1e})" for r in report))
    assert not failures, failures
    # three layers deep, bf16 storage alone costs 1e-2 .. 3e-2 on the gradients (the figures in brackets); the top
    # output, the bottom input gradient and the bottom layer's gradients must not need the storage rule
    assert not [n for n in excess if n.startswith(("top", "dX", "layer 0"))], excess


# ------------------------------------------------------------------------------------------------------------
# Sampled layers of a whole-model iteration.  All layers of the model are resident and one iteration runs
# (forward through every layer, loss head, backward through every layer).  For the first, the middle and the last
# layer the test takes what that layer was GIVEN in that iteration - its input rows and the gradient rows that
# reached it, both produced by the device's layers above / below, which the oracle cannot compute at this size -
# regenerates the layer's weights from its seed on the host, recomputes a sample of requests with the oracle and
# holds the layer's own outputs (output rows, saved activations, input gradient, KV-gradient accumulator, LoRA
# gradients) to it.  It is a per-layer check at depth; the chained checks whose oracle side never sees a device
# value are the three-layer chain above and the training-step tests.
# ------------------------------------------------------------------------------------------------------------
def _layer_sampled_check(model, n_decode, inference_share=None):
    import numpy as np
    from paper_2402_18789_amd import model_iter
    from oracle import layer as OL
    from oracle.maps import build_maps
    from workload import gen, CONFIGS
    from gpu_common import assert_close, to_np, TOL
    cfg_name, make_batch, _ = model_iter.MODELS[model]
    cfg, seed = CONFIGS[cfg_name], 0
    tol = TOL["bf16"]
    batch = make_batch(seed) if inference_share is None else make_batch(seed, inference_share)
    sample = gen.sample_requests(batch, n_decode)
    n_layers = cfg.n_layers
    which = (0, n_layers // 2, n_layers - 1)
    say("whole-model iteration %s (%d layers), layers %s checked on sampled requests" % (cfg_name, n_layers, which))
    r = model_iter.run(steps=1, warmup=1, seed=seed, model=model, inference_share=inference_share, capture_layers=which,
                       sample=sample)
    assert r["finite"]
    cap = r["captured"]
    ft_req, L = cap["ft_req"], cap["seq_len"]
    rows = gen.sample_token_rows(batch, sample)
    cpages, n_cp = _compact_pages(batch, sample)
    om = build_maps(sample, cpages, batch.page_size, n_cp)
    w = slice(ft_req.start_pos, ft_req.start_pos + ft_req.n_new)
    for n in which:
        c = cap["rows"][n]
        W, lo = gen.layer_weights(cfg, seed, n), gen.lora_weights(cfg, seed, n)
        o_pool = OL.KVPool(n_cp, cfg.page_size, cfg.kv_dim, dtype=np.float32)
        for q in sample:
            if q.start_pos:
                k, v = gen.kv_prefix(cfg, seed, n, q.seq_id, q.start_pos)
                sl = o_pool.slots(cpages[q.seq_id], q.start_pos)
                o_pool.k[sl], o_pool.v[sl] = k, v
        o_ft = OL.FtState(cfg, L)
        report = []
        y_o = OL.layer_forward_mixed(cfg, W, lo, om, to_np(c["x_in"])[rows], o_pool, {ft_req.seq_id: o_ft})
        assert_close("y", to_np(c["x_out"])[rows], y_o, tol, report)
        ft_d = cap["fts"][n]
        for name in ("q_cache", "x2", "gate", "up", "attn", "lse"):
            assert_close("saved " + name, to_np(getattr(ft_d, name))[w], getattr(o_ft, name)[w], tol, report)
        sl = o_pool.slots(cpages[ft_req.seq_id], L)
        grads = {}
        dX_o = OL.layer_backward_window(cfg, W, lo, o_ft, o_pool.k[sl].astype(np.float64), o_pool.v[sl].astype(np.float64),
                                        ft_req.start_pos, ft_req.n_new, to_np(c["dY"]), grads, need_dx=n > 0)
        if n > 0:
            assert_close("dX", to_np(c["dX"]), dX_o, tol, report)
        assert_close("dk_accum", to_np(ft_d.dk_accum), o_ft.dk_accum, tol, report)
        assert_close("dv_accum", to_np(ft_d.dv_accum), o_ft.dv_accum, tol, report)
        gg = cap["layers"][n].grads_numpy()
        for t in cfg.lora_targets:
            assert_close(f"dA[{t}]", gg[t][0], grads[t][0], tol, report)
            assert_close(f"dB[{t}]", gg[t][1], grads[t][1], tol, report)
        say("  layer %d: " % n + ", ".join(f"{k}={e:.1e}" for k, e in report))
    say("  iteration: %.1f ms (%d tokens, %d finetune), %.1f GB resident" % (
        r["ms_per_iteration"], r["config"]["tokens"], r["config"]["finetune_tokens"], r["resident_gb"]["allocated"]))
    del cap, r
    import gc
    import torch
    gc.collect()
    torch.cuda.empty_cache()


def test_whole_model_iteration_8b_layers_sampled():
    _layer_sampled_check("c3", 8)


@pytest.mark.parametrize("model,share", [("c4", None), ("c4", 0.25), ("c4", 0.9), ("c5", None)])
def test_whole_model_iteration_14b_32b_layers_sampled(model, share):
    """The 14B-shaped (48 layers, 185 GB resident) and 32B-shaped (64 layers, 269 GB) models the same way; the
    14B one also at the two ends of its inference-share sweep.  Minutes of set-up each: run on request,
    FLEXCO_BIG_MODELS=1 python -m pytest tests/test_gpu_model_iter.py -m gpu -k 14b_32b -s"""
    import os
    if os.environ.get("FLEXCO_BIG_MODELS") != "1":
        pytest.skip("set FLEXCO_BIG_MODELS=1 to build the 48- and 64-layer models")
    _layer_sampled_check(model, 4, share)


def test_library_layer_loop_equals_per_layer_calls():
    """flexco_model_forward / flexco_model_backward (the loops over the layers inside the library, odd and even
    numbers of layers, with and without an input gradient below the bottom layer) leave bit for bit what the
    same layers called one by one leave."""
    import numpy as np
    import torch
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from workload import gen, CONFIGS
    cfg = CONFIGS["c2_llama8b_layer"].with_(name="small_bf16", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408)
    seed = 5
    batch = gen.batch_scaled(seed, 9, 20, 500, [(0, 100, 100), (128, 64, 300)], [(64, 96, 160)])
    ft_req = [r for r in batch.requests if r.kind == 2][0]
    L = batch.seq_capacity[ft_req.seq_id]
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    hm = db.host_maps
    x = torch.from_numpy(gen.layer_input(cfg, seed, hm.T)).to("cuda", torch.bfloat16)
    dY0 = torch.from_numpy(gen.layer_input(cfg, seed, ft_req.n_new, tag="dy")).to("cuda", torch.bfloat16)
    pages = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")
    for N, need_dx0 in ((1, True), (2, False), (3, True)):
        say("library layer loop, %d layers, bottom input gradient %s" % (N, need_dx0))
        arena = HH.ParamArena(N * HH.lora_param_elems(cfg), torch.bfloat16)

        def fresh():
            ls = [HH.DeviceLayer(cfg, gen.layer_weights(cfg, seed, n), gen.lora_weights(cfg, seed, n)) for n in range(N)]
            ps = [HH.DevicePool(cfg, batch.num_pages) for _ in range(N)]
            for n, p in enumerate(ps):
                p.fill_random(seed + n)
            fs = [HH.DeviceFtState(cfg, L) for _ in range(N)]
            return ls, ps, fs
        ws = HH.Workspace(HH.c_cfg(cfg), hm.T, hm.n_parts, ft_req.n_new, L)
        # one by one
        ls, ps, fs = fresh()
        cur = x
        for n in range(N):
            out = torch.empty_like(x)
            B.flexco_layer_forward(ls[n].c, ls[n].w, ls[n].lora, db.maps, cur, out, ps[n].c, fs[n].c, ws.ptr, ws.bytes)
            cur = out
        y_ref = cur.clone()
        d = dY0.clone()
        for n in range(N - 1, -1, -1):
            dx = torch.empty_like(d) if (n > 0 or need_dx0) else None
            B.flexco_lora_bwd(ls[n].c, ls[n].w, ls[n].lora, ps[n].c, pages, len(pages), fs[n].c, ft_req.start_pos, ft_req.n_new,
                              d, dx, ws.ptr, ws.bytes)
            d = dx if dx is not None else d
        torch.cuda.synchronize()
        dx_ref = d.clone() if need_dx0 else None
        # the library's loops
        ls2, ps2, fs2 = fresh()
        arr, keep = B.make_model_layers([(ls2[n].w, ls2[n].lora, ps2[n].c, fs2[n].c) for n in range(N)])
        y2, tmp = torch.empty_like(x), torch.empty_like(x)
        B.flexco_model_forward(ls2[0].c, arr, N, db.maps, x, y2, tmp if N > 1 else None, ws.ptr, ws.bytes)
        dY, dtmp = dY0.clone(), torch.empty_like(dY0)
        where = B.flexco_model_backward(ls2[0].c, arr, N, pages, len(pages), ft_req.start_pos, ft_req.n_new, dY, dtmp, need_dx0,
                                        ws.ptr, ws.bytes)
        torch.cuda.synchronize()
        assert torch.equal(y2, y_ref)
        if need_dx0:
            assert where in (dY.data_ptr(), dtmp.data_ptr())
            assert torch.equal(dY if where == dY.data_ptr() else dtmp, dx_ref)
        else:
            assert where is None
        for n in range(N):
            for t in cfg.lora_targets:
                assert torch.equal(ls2[n].dA[t], ls[n].dA[t]) and torch.equal(ls2[n].dB[t], ls[n].dB[t]), (n, t)
            assert torch.equal(fs2[n].dk_accum, fs[n].dk_accum) and torch.equal(fs2[n].q_cache, fs[n].q_cache)
            assert torch.equal(ps2[n].k, ps[n].k) and torch.equal(ps2[n].v, ps[n].v)
        del arena
    # error paths: no layers; one buffer given twice
    with pytest.raises(B.FlexcoError):
        B.flexco_model_forward(ls2[0].c, arr, 0, db.maps, x, y2, tmp, ws.ptr, ws.bytes)
    with pytest.raises(B.FlexcoError):
        B.flexco_model_forward(ls2[0].c, arr, N, db.maps, x, y2, y2, ws.ptr, ws.bytes)
    with pytest.raises(B.FlexcoError):
        B.flexco_model_backward(ls2[0].c, arr, N, pages, len(pages), ft_req.start_pos, ft_req.n_new, dY, dY, True, ws.ptr, ws.bytes)


def test_adam_over_one_flat_parameter_buffer_equals_per_matrix_steps():
    """The bypass matrices of several layers carved from one flat buffer and updated by ONE flexco_adam_step call
    end up bit for bit where per-matrix calls put them."""
    import torch
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from workload import gen, CONFIGS
    cfg = CONFIGS["c2_llama8b_layer"].with_(name="small_bf16", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408,
                                           lora_rank=24)      # 24-row matrices: pieces that need their padding
    N = 3
    arena = HH.ParamArena(N * HH.lora_param_elems(cfg), torch.bfloat16)
    flat = [HH.DeviceLora(cfg, gen.lora_weights(cfg, 2, n), arena=arena) for n in range(N)]
    sep = [HH.DeviceLora(cfg, gen.lora_weights(cfg, 2, n)) for n in range(N)]
    assert arena.used == arena.param.numel()
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    for a, b in zip(flat, sep):
        for t in cfg.lora_targets:
            assert a.A[t].data_ptr() % 16 == 0 and a.dB[t].data_ptr() % 16 == 0
            for ga, gb in ((a.dA[t], b.dA[t]), (a.dB[t], b.dB[t])):
                gb.copy_(torch.randn(gb.shape, generator=g, device="cuda"))
                ga.copy_(gb)
    n = arena.used
    master = arena.param.float()
    m, v = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    state = []
    for b in sep:
        for t in cfg.lora_targets:
            for P, G in ((b.A[t], b.dA[t]), (b.Bm[t], b.dB[t])):
                state.append((P, P.float().clone(), G, torch.zeros_like(G), torch.zeros_like(G)))
    for step in (1, 2):
        B.flexco_adam_step(arena.param, master, arena.grad, m, v, n, 1, 1e-3, 0.9, 0.999, 1e-8, step)
        for P, M, G, m1, v1 in state:
            B.flexco_adam_step(P, M, G, m1, v1, P.numel(), 1, 1e-3, 0.9, 0.999, 1e-8, step)
    torch.cuda.synchronize()
    for a, b in zip(flat, sep):
        for t in cfg.lora_targets:
            assert torch.equal(a.A[t], b.A[t]) and torch.equal(a.Bm[t], b.Bm[t]), t
