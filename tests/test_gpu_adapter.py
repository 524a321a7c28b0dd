"""GPU parity of the bottleneck adapter bypass network (flexco_adapter_fwd / flexco_adapter_bwd) against
oracle/adapter.py: alone on a mixed batch's rows, and composed with the decoder layer in a two-layer stack
trained through token windows (Alg. 2) against the whole-sequence definition."""
import numpy as np
import pytest
import torch

import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH
from oracle import adapter as OA
from oracle import layer as OL
from workload import gen
from workload.configs import CONFIGS, KIND_FINETUNE
from gpu_common import TOL, assert_close, to_np

pytestmark = pytest.mark.gpu

C1 = CONFIGS["c1_tiny_f32"].with_(lora_targets=())
SMALL_BF16 = CONFIGS["c2_llama8b_layer"].with_(name="small_bf16_ad", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128,
                                               ffn=1408, lora_targets=())


def say(msg):
    print(msg, flush=True)


def adapter_weights(cfg, seed, layer, b):
    g = gen.rng(seed, cfg.name, layer, "adapter", b)
    wd = gen.storage_round(cfg, (g.standard_normal((b, cfg.hidden), dtype=np.float32) * np.float32(0.05)))
    wu = gen.storage_round(cfg, (g.standard_normal((cfg.hidden, b), dtype=np.float32) * np.float32(0.05)))
    return wd, wu


class DeviceAdapter:
    def __init__(self, cfg, wd, wu):
        dt = HH.TORCH_DTYPE[cfg.dtype]
        self.wd, self.wu = torch.from_numpy(wd).to("cuda", dt), torch.from_numpy(wu).to("cuda", dt)
        self.dwd = torch.zeros(wd.shape, dtype=torch.float32, device="cuda")
        self.dwu = torch.zeros(wu.shape, dtype=torch.float32, device="cuda")
        self.c = B.Adapter(wd.shape[0], self.wd.data_ptr(), self.wu.data_ptr(), self.dwd.data_ptr(), self.dwu.data_ptr())


@pytest.mark.parametrize("cfg,b", [(C1, 8), (SMALL_BF16, 64), (SMALL_BF16, 24)])
def test_adapter_alone_on_a_mixed_batch(cfg, b):
    say(f"adapter alone: {cfg.name}, bottleneck {b}")
    tol = TOL[cfg.dtype]
    batch = gen.with_adapters(gen.batch_scaled(3, 9, 5, 300, [(0, 37, 37), (64, 50, 130)], [(40, 33, 90)]), [0, -1])
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    hm = db.host_maps
    T = hm.T
    ft_req = [r for r in batch.requests if r.kind == KIND_FINETUNE][0]
    L = batch.seq_capacity[ft_req.seq_id]
    wd, wu = adapter_weights(cfg, 1, 0, b)
    ad = DeviceAdapter(cfg, wd, wu)
    dt = HH.TORCH_DTYPE[cfg.dtype]
    x = gen.layer_input(cfg, 1, T, tag="adapter_x")
    y_d = torch.from_numpy(x).to("cuda", dt)
    saved = torch.zeros((L, cfg.hidden), dtype=dt, device="cuda")
    nbytes = B.flexco_adapter_workspace_bytes(HH.DTYPE_CODE[cfg.dtype], cfg.hidden, b, T, L)
    ws = torch.empty(nbytes // 4 + 1, dtype=torch.float32, device="cuda")
    B.flexco_adapter_fwd(HH.DTYPE_CODE[cfg.dtype], cfg.hidden, ad.c, db.maps, y_d, saved, L, ws, ws.numel() * 4)
    torch.cuda.synchronize()
    om = db.numpy()
    rows = om["tok_adapter"] >= 0
    assert 0 < rows.sum() < T
    y_o = OA.forward(x.astype(np.float64), wd.astype(np.float64), wu.astype(np.float64), rows)
    got = to_np(y_d)
    assert_close("adapter forward", got, y_o, tol)
    assert np.array_equal(got[~rows], x[~rows].astype(np.float64))            # rows without the adapter: untouched
    t0 = int(hm.ft_tok0)
    w = slice(ft_req.start_pos, ft_req.start_pos + ft_req.n_new)
    assert np.array_equal(to_np(saved)[w], x[t0:t0 + ft_req.n_new].astype(np.float64))
    # backward over the window in two pieces, from its end
    dy = gen.layer_input(cfg, 1, ft_req.n_new, tag="adapter_dy")
    x_w = x[t0:t0 + ft_req.n_new].astype(np.float64)
    dx_o, dwd_o, dwu_o = OA.backward(x_w, wd.astype(np.float64), wu.astype(np.float64), dy.astype(np.float64))
    dx_g = np.zeros_like(dx_o)
    l = ft_req.n_new
    for s in (13, l - 13):
        dY_d = torch.from_numpy(dy[l - s:l]).to("cuda", dt)
        B.flexco_adapter_bwd(HH.DTYPE_CODE[cfg.dtype], cfg.hidden, ad.c, saved, L, ft_req.start_pos + l - s, s, dY_d, ws,
                             ws.numel() * 4)
        torch.cuda.synchronize()
        dx_g[l - s:l] = to_np(dY_d)
        l -= s
    assert_close("adapter dX", dx_g, dx_o, tol)
    assert_close("adapter dW_down", to_np(ad.dwd), dwd_o, tol)
    assert_close("adapter dW_up", to_np(ad.dwu), dwu_o, tol)


@pytest.mark.parametrize("cfg,b,L,fwd,bwd", [(C1, 8, 96, (40, 56), (30, 66)), (SMALL_BF16, 32, 384, (150, 234), (120, 264)),
                                             (SMALL_BF16, 64, 384, (150, 234), (120, 264))])
def test_two_layers_with_adapters_trained_through_token_windows(cfg, b, L, fwd, bwd):
    """Layer, adapter, layer, adapter; forward in windows through the caches, backward in other windows, against
    the whole-sequence definition composed from the two oracles (frozen layers: only the adapters train)."""
    say(f"two layers with adapters: {cfg.name}")
    tol = TOL[cfg.dtype]
    seed, N = 4, 2
    dt = HH.TORCH_DTYPE[cfg.dtype]
    code = HH.DTYPE_CODE[cfg.dtype]
    Ws = [gen.layer_weights(cfg, seed, n) for n in range(N)]
    ads_np = [adapter_weights(cfg, seed, n, b) for n in range(N)]
    x = gen.layer_input(cfg, seed, L, tag="x_stack")
    # ---- oracle: whole sequence ----
    h, inputs, ad_in = x.astype(np.float64), [], []
    for n in range(N):
        inputs.append(h)
        y = OL.layer_forward_seq(cfg, Ws[n], None, h)["y"]
        ad_in.append(y)
        h = OA.forward(y, ads_np[n][0].astype(np.float64), ads_np[n][1].astype(np.float64))
    target = gen.loss_targets(cfg, seed, L).astype(np.float64)
    _, dY = OL.mse_loss_grad(h, target)
    dY = gen.storage_round(cfg, (dY * L * cfg.hidden).astype(np.float32)).astype(np.float64)
    grads_o, d = [None] * N, dY
    for n in range(N - 1, -1, -1):
        d, gd, gu = OA.backward(ad_in[n], ads_np[n][0].astype(np.float64), ads_np[n][1].astype(np.float64), d)
        grads_o[n] = (gd, gu)
        d, _, _, _ = OL.layer_backward_seq(cfg, Ws[n], {}, inputs[n], d)
    # ---- GPU: token level ----
    devs = [HH.DeviceLayer(cfg, Ws[n], None) for n in range(N)]
    ads = [DeviceAdapter(cfg, *ads_np[n]) for n in range(N)]
    fts = [HH.DeviceFtState(cfg, L) for _ in range(N)]
    saved = [torch.zeros((L, cfg.hidden), dtype=dt, device="cuda") for _ in range(N)]
    y_top = torch.zeros((L, cfg.hidden), dtype=dt, device="cuda")
    l = 0
    batch = None
    for s in fwd:
        batch = gen.mixed_batch(16, seed, decode_ctx=(), prefill=(), finetune=[(l, s, L)])
        if l == 0:
            pools = [HH.DevicePool(cfg, batch.num_pages) for _ in range(N)]
            pages = batch.seq_pages[0]
        batch.seq_pages[0] = pages
        db = HH.DeviceBatch(cfg, batch.requests, {0: pages}, pools[0].num_pages)
        ws = HH.Workspace(devs[0].c, s, db.host_maps.n_parts)
        aws = torch.empty(B.flexco_adapter_workspace_bytes(code, cfg.hidden, b, L, L) // 4 + 1, dtype=torch.float32, device="cuda")
        cur = torch.from_numpy(x[l:l + s]).to("cuda", dt)
        for n in range(N):
            out = torch.empty_like(cur)
            B.flexco_layer_forward(devs[n].c, devs[n].w, None, db.maps, cur, out, pools[n].c, fts[n].c, ws.ptr, ws.bytes)
            B.flexco_adapter_fwd(code, cfg.hidden, ads[n].c, db.maps, out, saved[n], L, aws, aws.numel() * 4)
            cur = out
        y_top[l:l + s] = cur
        l += s
    torch.cuda.synchronize()
    assert_close("stack output", to_np(y_top), h, tol)
    pages_d = torch.from_numpy(np.asarray(pages, dtype=np.int32)).to("cuda")
    for f in fts:
        f.zero_accum()
    report = []
    rnd = lambda a: np.asarray(gen.storage_round(cfg, np.asarray(a, dtype=np.float32)), dtype=np.float64)
    aws = torch.empty(B.flexco_adapter_workspace_bytes(code, cfg.hidden, b, L, L) // 4 + 1, dtype=torch.float32, device="cuda")

    def gpu_stage(n, src, saved_rows):
        """adapter n's backward, then layer n's, over the backward windows from the end, on the gradient rows
        `src` -> (gradient below the adapter, gradient below the layer)"""
        l = L
        d_ad, d_layer = np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden))
        for s_ in bwd:
            ws = HH.Workspace(devs[0].c, 0, 0, s_, l)
            d_d = torch.from_numpy(np.ascontiguousarray(src[l - s_:l], dtype=np.float32)).to("cuda", dt)
            B.flexco_adapter_bwd(code, cfg.hidden, ads[n].c, saved_rows, L, l - s_, s_, d_d, aws, aws.numel() * 4)
            dX_d = torch.empty_like(d_d)
            B.flexco_lora_bwd(devs[n].c, devs[n].w, None, pools[n].c, pages_d, len(pages), fts[n].c, l - s_, s_, d_d, dX_d,
                              ws.ptr, ws.bytes)
            torch.cuda.synchronize()
            d_ad[l - s_:l], d_layer[l - s_:l] = to_np(d_d), to_np(dX_d)
            l -= s_
        return d_ad, d_layer

    if cfg.dtype == "f32":
        # the whole chain on the device's own values against the whole-sequence definition
        src = dY
        for n in range(N - 1, -1, -1):
            _, src = gpu_stage(n, src, saved[n])
        assert_close("dX of the stack", src, d, tol, report)
        for n in range(N):
            assert_close(f"layer {n} dW_down", to_np(ads[n].dwd), grads_o[n][0], tol, report)
            assert_close(f"layer {n} dW_up", to_np(ads[n].dwu), grads_o[n][1], tol, report)
    else:
        # bf16.  The ReLU's backward mask is an integer decision (sign of x W_down^T) taken from stored rows; two
        # correct implementations whose stored rows differ in the last bf16 bit take it differently for the few
        # units that sit at zero, and one such unit moves its row of dX by several percent.  Both sides must
        # therefore take the decision on the same values: every stage of the backward chain (adapter n, then
        # layer n, from the top) runs on the device with the ORACLE's values as its inputs - the oracle's
        # adapter-input rows (rounded to the storage type) in place of the rows the device stored, the oracle's
        # gradient rows from the stage above - and is held to the oracle's result for that stage at the bf16 bar.
        # The oracle never sees a device value.  (The chain on the device's own values end to end is the fp32
        # case above, where the decisions coincide.)
        src = dY                                        # already rounded to the storage type
        for n in range(N - 1, -1, -1):
            x_ad = rnd(ad_in[n])
            forced = torch.from_numpy(np.ascontiguousarray(x_ad, dtype=np.float32)).to("cuda", dt)
            assert_close(f"layer {n} stored adapter input", to_np(saved[n]), ad_in[n], tol, report)
            d_ad_g, d_layer_g = gpu_stage(n, src, forced)
            d_ad_o, gd, gu = OA.backward(x_ad, ads_np[n][0].astype(np.float64), ads_np[n][1].astype(np.float64), src)
            d_layer_o, _, _, _ = OL.layer_backward_seq(cfg, Ws[n], {}, inputs[n], rnd(d_ad_o))
            assert_close(f"layer {n} adapter dX", d_ad_g, d_ad_o, tol, report)
            assert_close(f"layer {n} dW_down", to_np(ads[n].dwd), gd, tol, report)
            assert_close(f"layer {n} dW_up", to_np(ads[n].dwu), gu, tol, report)
            assert_close(f"layer {n} dX", d_layer_g, d_layer_o, tol, report)
            src = rnd(d_layer_o)
    say("  " + ", ".join(f"{n}={e:.1e}" for n, e in report))


def test_adapter_error_paths():
    cfg = SMALL_BF16
    wd, wu = adapter_weights(cfg, 0, 0, 16)
    ad = DeviceAdapter(cfg, wd, wu)
    b = gen.batch_scaled(1, 2, 3, 40, [], [(0, 16, 16)])
    db = HH.DeviceBatch(cfg, b.requests, b.seq_pages, b.num_pages)
    y = torch.zeros((db.host_maps.T, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    saved = torch.zeros((16, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 16, dtype=torch.float32, device="cuda")
    with pytest.raises(B.FlexcoError) as e:                        # workspace too small
        B.flexco_adapter_fwd(1, cfg.hidden, ad.c, db.maps, y, saved, 16, ws, 16)
    assert e.value.code == B.FLEXCO_EWORKSPACE
    with pytest.raises(B.FlexcoError) as e:                        # state shorter than the window
        B.flexco_adapter_fwd(1, cfg.hidden, ad.c, db.maps, y, saved, 8, ws, ws.numel() * 4)
    assert e.value.code == B.FLEXCO_ESHAPE
    wide = B.Adapter(65, ad.c.w_down, ad.c.w_up, ad.c.dw_down, ad.c.dw_up)
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_adapter_fwd(1, cfg.hidden, wide, db.maps, y, saved, 16, ws, ws.numel() * 4)
    assert e.value.code == B.FLEXCO_ESHAPE
    nograd = B.Adapter(16, ad.c.w_down, ad.c.w_up, None, None)
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_adapter_bwd(1, cfg.hidden, nograd, saved, 16, 0, 16, y[:16], ws, ws.numel() * 4)
    assert e.value.code == B.FLEXCO_EINVAL
    with pytest.raises(B.FlexcoError) as e:                        # window beyond the sequence
        B.flexco_adapter_bwd(1, cfg.hidden, ad.c, saved, 16, 8, 16, y[:16], ws, ws.numel() * 4)
    assert e.value.code == B.FLEXCO_ESHAPE
