"""GPU parity of the (IA)^3 bypass network (Sec. 4.1) through the C ABI: mixed batches over several
iterations (decode and prefill requests with and without the adapter, finetune windows), then the
token-window backward pass, against oracle/ia3.py on the same seeded inputs."""
import numpy as np
import pytest
import torch

import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH
from oracle import ia3 as OI
from oracle import layer as OL
from oracle.maps import build_maps
from workload import gen
from workload.configs import CONFIGS, KIND_FINETUNE
from gpu_common import TOL, assert_close, to_np

pytestmark = pytest.mark.gpu

C1 = CONFIGS["c1_tiny_f32"].with_(lora_targets=())
C2 = CONFIGS["c2_llama8b_layer"]
SMALL_BF16 = C2.with_(name="small_bf16_ia3", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408, lora_targets=())
SMALL_BF16_G5 = C2.with_(name="small_bf16_g5_ia3", hidden=640, n_q_heads=10, n_kv_heads=2, head_dim=128, ffn=1152,
                         lora_targets=(), qkv_bias=True, rms_eps=1e-6, rope_theta=1e6)


def say(msg):
    print(msg, flush=True)


def run_case(cfg, batch0, ft_window, prefill_chunk, bwd_windows, seed, need_dx=True):
    tol = TOL[cfg.dtype]
    report = []
    W = gen.layer_weights(cfg, seed, 0)
    ia3 = gen.ia3_weights(cfg, seed, 0)
    dev = HH.DeviceLayer(cfg, W, None)
    dia = HH.DeviceIa3(cfg, ia3)
    ft_seq = [r.seq_id for r in batch0.requests if r.kind == KIND_FINETUNE][0]
    L = batch0.seq_capacity[ft_seq]
    o_pool = OL.KVPool(batch0.num_pages, cfg.page_size, cfg.kv_dim)
    d_pool = HH.DevicePool(cfg, batch0.num_pages)
    o_ft, d_ft = OI.Ia3FtState(cfg, L), HH.DeviceFtState(cfg, L, ia3=True)
    for r in batch0.requests:                       # cached prefixes of the inference requests
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            sl = o_pool.slots(batch0.seq_pages[r.seq_id], r.start_pos)
            o_pool.k[sl], o_pool.v[sl] = k, v
            d_pool.write_rows(batch0.seq_pages[r.seq_id], k, v)
    dt = HH.TORCH_DTYPE[cfg.dtype]
    batch, it = batch0, 0
    y_ft = np.zeros((L, cfg.hidden))
    while any(r.kind == KIND_FINETUNE for r in batch.requests):
        say(f"  forward iteration {it}: T={batch.n_tokens}")
        x = gen.layer_input(cfg, seed, batch.n_tokens, tag=f"x{it}")
        db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
        ws = HH.Workspace(dev.c, db.host_maps.T, db.host_maps.n_parts)
        x_d = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda", dt)
        y_d = torch.empty_like(x_d)
        B.flexco_layer_forward_ia3(dev.c, dev.w, dia.c, db.maps, x_d, y_d, d_pool.c, d_ft.c, ws.ptr, ws.bytes)
        torch.cuda.synchronize()
        om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
        y_o = OI.forward_mixed(cfg, W, ia3, om, x, o_pool, {ft_seq: o_ft})
        assert_close(f"y it{it}", to_np(y_d), y_o, tol, report)
        for r, off in zip(batch.requests, np.cumsum([0] + [q.n_new for q in batch.requests])):
            kg, vg = d_pool.read_rows(batch.seq_pages[r.seq_id], r.n_new, r.start_pos)
            sl = o_pool.slots(batch.seq_pages[r.seq_id], r.start_pos + r.n_new)[r.start_pos:]
            assert_close(f"K append it{it}", kg, o_pool.k[sl], tol)
            assert_close(f"V append it{it}", vg, o_pool.v[sl], tol)
            if r.kind == KIND_FINETUNE:
                y_ft[r.start_pos:r.start_pos + r.n_new] = y_o[off:off + r.n_new]
        batch = gen.advance(batch, prefill_chunk=prefill_chunk, ft_window=ft_window)
        it += 1
    for name in ("q_cache", "x", "x2", "gate", "up", "attn", "k0", "v0"):
        assert_close("saved " + name, to_np(getattr(d_ft, name)), getattr(o_ft, name), tol, report)
    assert_close("saved lse", to_np(d_ft.lse), o_ft.lse, tol, report)
    # backward: MSE to seeded targets on the finetune sequence's output, the oracle's dY on both sides
    target = gen.loss_targets(cfg, seed, L).astype(np.float64)
    _, dY = OL.mse_loss_grad(y_ft, target)
    dY = gen.storage_round(cfg, (dY * L * cfg.hidden).astype(np.float32)).astype(np.float64)
    pages = batch0.seq_pages[ft_seq]
    pages_d = torch.from_numpy(np.asarray(pages, dtype=np.int32)).to("cuda")
    slots = o_pool.slots(pages, L)
    grads_o = {}
    dia.zero_grads()
    d_ft.zero_accum()
    dX_g, dX_o = np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden))
    l = L
    for s in bwd_windows:
        say(f"  backward window [{l - s}, {l})")
        ws = HH.Workspace(dev.c, 0, 0, s, l)
        dY_d = torch.from_numpy(np.ascontiguousarray(dY[l - s:l], dtype=np.float32)).to("cuda", dt)
        dX_d = torch.empty_like(dY_d) if need_dx else None
        B.flexco_ia3_bwd(dev.c, dev.w, dia.c, d_pool.c, pages_d, len(pages), d_ft.c, l - s, s, dY_d, dX_d, ws.ptr, ws.bytes)
        torch.cuda.synchronize()
        o = OI.backward_window(cfg, W, ia3, o_ft, o_pool.k[slots[:l]], o_pool.v[slots[:l]], l - s, s, dY[l - s:l], grads_o,
                               need_dx)
        if need_dx:
            dX_g[l - s:l], dX_o[l - s:l] = to_np(dX_d), o
        l -= s
    assert l == 0
    if need_dx:
        assert_close("dX", dX_g, dX_o, tol, report)
    assert_close("dk_accum", to_np(d_ft.dk_accum), o_ft.dk_accum, tol, report)
    assert_close("dv_accum", to_np(d_ft.dv_accum), o_ft.dv_accum, tol, report)
    assert_close("dl_ff", to_np(dia.dl["ff"]), grads_o["ff"], tol, report)
    assert_close("dl_v", to_np(dia.dl["v"]), grads_o["v"], tol, report)
    assert_close("dl_k", to_np(dia.dl["k"]), grads_o["k"], tol, report)
    say("  " + ", ".join(f"{n}={e:.1e}" for n, e in report))
    return report


def test_ia3_c1_fp32():
    say("(IA)^3 layer, c1 shape fp32")
    b = gen.with_adapters(gen.batch_c1(0), [0, -1])
    run_case(C1, b, ft_window=32, prefill_chunk=32, bwd_windows=[32, 32], seed=0)


def test_ia3_c1_fp32_uneven_windows_without_input_grad():
    say("(IA)^3 layer, c1 shape fp32, uneven windows, no input gradient")
    b = gen.with_adapters(gen.mixed_batch(16, 3, decode_ctx=(5, 16, 33), prefill=[(0, 20, 40)], finetune=[(0, 7, 50)]), [-1, 0])
    run_case(C1, b, ft_window=19, prefill_chunk=11, bwd_windows=[1, 30, 19], seed=3, need_dx=False)


def test_ia3_small_bf16():
    say("(IA)^3 layer, small bf16")
    b = gen.with_adapters(gen.batch_scaled(7, 10, 3, 600, [(0, 130, 130), (256, 64, 400)], [(0, 100, 260)]), [0, -1, 0])
    run_case(SMALL_BF16, b, ft_window=160, prefill_chunk=70, bwd_windows=[60, 200], seed=7)


def test_ia3_small_bf16_group5_bias():
    say("(IA)^3 layer, small bf16, kv group of 5, qkv bias")
    b = gen.with_adapters(gen.batch_scaled(5, 7, 17, 333, [(0, 40, 40)], [(0, 100, 164)]), [0])
    run_case(SMALL_BF16_G5, b, ft_window=64, prefill_chunk=40, bwd_windows=[33, 131], seed=5)


def test_ia3_inference_only_batch():
    """No finetune request (ft state = NULL): requests served with the adapter and base-model requests side by side."""
    cfg, seed = SMALL_BF16, 11
    say("(IA)^3 layer, inference-only batch")
    batch = gen.with_adapters(gen.mixed_batch(16, seed, decode_ctx=(1, 16, 17, 130), prefill=[(0, 33, 70), (48, 20, 90)]), [0, -1])
    W, ia3 = gen.layer_weights(cfg, seed, 0), gen.ia3_weights(cfg, seed, 0)
    dev, dia = HH.DeviceLayer(cfg, W, None), HH.DeviceIa3(cfg, ia3)
    o_pool, d_pool = OL.KVPool(batch.num_pages, cfg.page_size, cfg.kv_dim), HH.DevicePool(cfg, batch.num_pages)
    for r in batch.requests:
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            sl = o_pool.slots(batch.seq_pages[r.seq_id], r.start_pos)
            o_pool.k[sl], o_pool.v[sl] = k, v
            d_pool.write_rows(batch.seq_pages[r.seq_id], k, v)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    ws = HH.Workspace(dev.c, db.host_maps.T, db.host_maps.n_parts)
    x = gen.layer_input(cfg, seed, batch.n_tokens)
    x_d = torch.from_numpy(x).to("cuda", torch.bfloat16)
    y_d = torch.empty_like(x_d)
    B.flexco_layer_forward_ia3(dev.c, dev.w, dia.c, db.maps, x_d, y_d, d_pool.c, None, ws.ptr, ws.bytes)
    torch.cuda.synchronize()
    om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
    y_o = OI.forward_mixed(cfg, W, ia3, om, x, o_pool, None)
    assert_close("y", to_np(y_d), y_o, TOL["bf16"])
    # the base-model requests' rows equal a run without any adapter, bit for bit
    ones = HH.DeviceIa3(cfg, {k: np.ones_like(v) for k, v in ia3.items()})
    d_pool2 = HH.DevicePool(cfg, batch.num_pages)
    d_pool2.k.copy_(d_pool.k)
    d_pool2.v.copy_(d_pool.v)
    y2 = torch.empty_like(x_d)
    B.flexco_layer_forward_ia3(dev.c, dev.w, ones.c, db.maps, x_d, y2, d_pool2.c, None, ws.ptr, ws.bytes)
    torch.cuda.synchronize()
    base_rows = om["tok_adapter"] < 0
    assert base_rows.any() and (~base_rows).any()
    assert np.array_equal(to_np(y_d)[base_rows], to_np(y2)[base_rows])
    assert not np.array_equal(to_np(y_d)[~base_rows], to_np(y2)[~base_rows])


def test_ia3_error_paths():
    cfg = SMALL_BF16
    W = gen.layer_weights(cfg, 0, 0)
    dev = HH.DeviceLayer(cfg, W, None)
    dia = HH.DeviceIa3(cfg, gen.ia3_weights(cfg, 0, 0))
    b = gen.batch_scaled(1, 2, 3, 40, [], [(0, 16, 16)])
    pool = HH.DevicePool(cfg, b.num_pages)
    db = HH.DeviceBatch(cfg, b.requests, b.seq_pages, b.num_pages)
    ws = HH.Workspace(dev.c, db.host_maps.T, db.host_maps.n_parts, 16, 16)
    x = torch.zeros((db.host_maps.T, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    ft_plain = HH.DeviceFtState(cfg, 16)                       # no saved_k0 / saved_v0
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_layer_forward_ia3(dev.c, dev.w, dia.c, db.maps, x, y, pool.c, ft_plain.c, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EINVAL
    with pytest.raises(B.FlexcoError) as e:                    # ia3 NULL
        B.flexco_layer_forward_ia3(dev.c, dev.w, None, db.maps, x, y, pool.c, ft_plain.c, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EINVAL
    lora_cfg = HH.c_cfg(C2.with_(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408))
    ft = HH.DeviceFtState(cfg, 16, ia3=True)
    with pytest.raises(B.FlexcoError) as e:                    # a configuration with LoRA targets
        B.flexco_layer_forward_ia3(lora_cfg, dev.w, dia.c, db.maps, x, y, pool.c, ft.c, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EUNSUPPORTED
    nograd = B.Ia3(dia.c.l_k, dia.c.l_v, dia.c.l_ff, None, None, None)
    pages_d = torch.from_numpy(np.asarray(b.seq_pages[2], dtype=np.int32)).to("cuda")
    with pytest.raises(B.FlexcoError) as e:                    # backward without gradient vectors
        B.flexco_ia3_bwd(dev.c, dev.w, nograd, pool.c, pages_d, len(pages_d), ft.c, 0, 16, x[:16], y[:16], ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EINVAL
