"""GPU-vs-oracle parity of the loss head (final norm, LM head, next-token cross-entropy and its gradient)
and of the Adam update, through the C ABI.  Same bar as the layer: 1e-4 (fp32), 2e-2 (bf16) max
relative error per tensor."""
import numpy as np
import pytest
import torch

from workload import gen, CONFIGS

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from oracle import train as OT
    from gpu_common import to_np, TOL, assert_close

C1 = CONFIGS["c1_tiny_f32"]


def run_loss(dtype, n, H, V, seed, ignore=()):
    cfg = C1.with_(dtype=dtype)
    g = gen.rng(seed, "gputrain", dtype, n, H, V)
    x = gen.storage_round(cfg, g.standard_normal((n, H), dtype=np.float32))
    gain = gen.storage_round(cfg, (1.0 + 0.05 * g.standard_normal(H)).astype(np.float32))
    w = gen.storage_round(cfg, (0.05 * g.standard_normal((V, H))).astype(np.float32))
    y = g.integers(0, V, n).astype(np.int32)
    for k, i in enumerate(ignore):
        y[i] = -1 if k % 2 == 0 else V + k        # no next token: negative, or outside the vocabulary
    scale = 1.0 / (n + 3)
    loss_o, dx_o = OT.generative_loss(x.astype(np.float64), gain.astype(np.float64), w.astype(np.float64), y, scale, 1e-5)
    dt = HH.TORCH_DTYPE[dtype]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dt)
    x_d, g_d, w_d = dev(x), dev(gain), dev(w)
    y_d = torch.from_numpy(y).to("cuda")
    head = B.LmHead(H, V, HH.DTYPE_CODE[dtype], 1e-5, g_d.data_ptr(), w_d.data_ptr())
    nbytes = B.flexco_lm_loss_workspace_bytes(head, n)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    loss_d = torch.full((1,), 0.25, dtype=torch.float32, device="cuda")     # the call adds to what is there
    dx_d = torch.empty_like(x_d)
    B.flexco_lm_loss(head, x_d, y_d, n, scale, loss_d, dx_d, ws, nbytes)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    got = float(loss_d.item()) - 0.25
    assert abs(got - loss_o) <= tol * abs(loss_o), (got, loss_o)
    assert_close("dx", to_np(dx_d), dx_o, tol)
    for i in ignore:
        assert np.abs(to_np(dx_d)[i]).max() == 0.0
    return got, loss_o


@pytest.mark.parametrize("dtype,n,H,V,ignore", [("f32", 37, 256, 1003, (5,)), ("f32", 4, 64, 50, ()),
                                                ("bf16", 70, 512, 4104, (0, 69)), ("bf16", 33, 256, 1001, ()),
                                                ("bf16", 1, 256, 2048, ())])
def test_loss_head(dtype, n, H, V, ignore):
    print(f"loss head {dtype} n={n} H={H} V={V}", flush=True)
    run_loss(dtype, n, H, V, seed=1, ignore=ignore)


def test_loss_head_llama_vocabulary():
    """The 8B shape's head: hidden 4096, vocabulary 128256, a window of 48 rows."""
    print("loss head bf16 at hidden 4096, vocabulary 128256", flush=True)
    run_loss("bf16", 48, 4096, 128256, seed=2, ignore=(47,))


def test_loss_head_qwen_vocabulary():
    """The 14B / 32B shapes' head: hidden 5120, vocabulary 152064, a window of 40 rows."""
    print("loss head bf16 at hidden 5120, vocabulary 152064", flush=True)
    run_loss("bf16", 40, 5120, 152064, seed=3, ignore=(0, 39))


def test_loss_head_window_of_600_rows_takes_the_large_input_gradient_tile():
    """dH = dZ W of 600 rows at hidden 1024, vocabulary 32768: 256 x 256 tiles with K cut over 16 blocks (the plan says so),
    the last row tile ragged, the partial sums added by the reduction kernel."""
    n, H, V = 600, 1024, 32768
    assert B.flexco_gemm_plan(n, H, V, 1, 16 * n * H) == [(256, 256, H, 16, 2)]
    print(f"loss head bf16 n={n} H={H} V={V}", flush=True)
    run_loss("bf16", n, H, V, seed=4, ignore=(0, 599))


def test_loss_head_all_rows_ignored_and_errors():
    cfg = C1
    H, V, n = 64, 40, 3
    x = torch.zeros((n, H), device="cuda")
    gain = torch.ones(H, device="cuda")
    w = torch.zeros((V, H), device="cuda")
    head = B.LmHead(H, V, 0, 1e-5, gain.data_ptr(), w.data_ptr())
    nbytes = B.flexco_lm_loss_workspace_bytes(head, n)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    y = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    dx = torch.ones((n, H), device="cuda")
    B.flexco_lm_loss(head, x, y, n, 1.0, loss, dx, ws, nbytes)
    torch.cuda.synchronize()
    assert float(loss.item()) == 0.0 and float(dx.abs().max().item()) == 0.0
    with pytest.raises(B.FlexcoError):
        B.flexco_lm_loss(head, x, y, n, 1.0, loss, dx, ws, 16)       # workspace too small
    B.flexco_lm_loss(head, x, y, 0, 1.0, loss, dx, ws, nbytes)       # empty window: nothing to do


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_adam_steps(dtype):
    cfg = C1.with_(dtype=dtype)
    n = 4099
    g = gen.rng(3, "gputrain", "adam", dtype)
    p0 = gen.storage_round(cfg, (0.02 * g.standard_normal(n)).astype(np.float32))
    dt = HH.TORCH_DTYPE[dtype]
    p_d = torch.from_numpy(p0).to("cuda", dt)
    master = torch.from_numpy(p0).to("cuda", torch.float32) if dtype == "bf16" else None
    m_d, v_d = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    p_o, m_o, v_o = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, 6):
        grad = (g.standard_normal(n) * 10.0 ** g.uniform(-4, 0, n)).astype(np.float32)
        B.flexco_adam_step(p_d, master, torch.from_numpy(grad).to("cuda"), m_d, v_d, n, HH.DTYPE_CODE[dtype], 1e-3, 0.9, 0.999, 1e-8,
                           step)
        p_o, m_o, v_o = OT.adam_step(p_o, grad.astype(np.float64), m_o, v_o, step, 1e-3)
    torch.cuda.synchronize()
    # the optimizer state is fp32 whatever the parameters' storage type
    assert_close("m", to_np(m_d), m_o, TOL["f32"])
    assert_close("v", to_np(v_d), v_o, TOL["f32"])
    if master is not None:
        assert_close("master", to_np(master), p_o, TOL["f32"])
    assert_close("param", to_np(p_d), p_o, TOL[dtype])
    with pytest.raises(B.FlexcoError):
        B.flexco_adam_step(p_d, master, m_d, m_d, v_d, n, HH.DTYPE_CODE[dtype], 1e-3, 0.9, 0.999, 1e-8, 0)


# ------------------------------------------------------------------------------------------
# Alg. 2 end to end: co-served forward windows through a stack of layers, the generative loss per
# window, token-level backward through the stack from the top, Adam -- against the sequence-level
# step written out as its definition (Sec. 6.1: the two are the same computation)
# ------------------------------------------------------------------------------------------
def run_training_step(cfg, n_layers, batch0, ft_window, prefill_chunk, bwd_windows, V, seed, lr, adam):
    from gpu_common import Case
    from workload.configs import KIND_FINETUNE
    tol = TOL[cfg.dtype]
    dt = HH.TORCH_DTYPE[cfg.dtype]
    ft_seq = [r.seq_id for r in batch0.requests if r.kind == KIND_FINETUNE][0]
    L, H = batch0.seq_capacity[ft_seq], cfg.hidden
    assert sum(bwd_windows) == L
    g = gen.rng(seed, "gputrain", "e2e", cfg.name, n_layers)
    x_seq = gen.storage_round(cfg, g.standard_normal((L, H), dtype=np.float32))
    gain = gen.storage_round(cfg, (1.0 + 0.05 * g.standard_normal(H)).astype(np.float32))
    w_lm = gen.storage_round(cfg, (0.05 * g.standard_normal((V, H))).astype(np.float32))
    targets = g.integers(0, V, L).astype(np.int32)
    targets[-1] = -1                                           # the last position has no next token
    layers = [gen.layer_weights(cfg, seed, n) for n in range(n_layers)]
    loras = [gen.lora_weights(cfg, seed, n, b_std=0.02) for n in range(n_layers)]
    cases = [Case(cfg, batch0, seed=seed, layer=n, weights=layers[n], lora=loras[n]) for n in range(n_layers)]

    g_d = torch.from_numpy(gain).to("cuda", dt)
    w_d = torch.from_numpy(w_lm).to("cuda", dt)
    head = B.LmHead(H, V, HH.DTYPE_CODE[cfg.dtype], cfg.rms_eps, g_d.data_ptr(), w_d.data_ptr())
    hb = B.flexco_lm_loss_workspace_bytes(head, L)
    hws = torch.empty(hb, dtype=torch.uint8, device="cuda")
    loss_d = torch.zeros(1, dtype=torch.float32, device="cuda")
    dtop = torch.zeros((L, H), dtype=dt, device="cuda")
    tgt_d = torch.from_numpy(targets).to("cuda")

    # ---- forward: iterations of the mixed batch until the finetune sequence is through ----------------
    batch, it = batch0, 0
    while any(r.kind == KIND_FINETUNE for r in batch.requests):
        x = gen.layer_input(cfg, seed, batch.n_tokens, tag=f"e2e{it}")
        offs = np.cumsum([0] + [r.n_new for r in batch.requests])
        ft = [(r, int(o)) for r, o in zip(batch.requests, offs) if r.kind == KIND_FINETUNE][0]
        r, off = ft
        print(f"  forward iteration {it}: T={batch.n_tokens}, finetune rows [{r.start_pos}, {r.start_pos + r.n_new})", flush=True)
        x[off:off + r.n_new] = x_seq[r.start_pos:r.start_pos + r.n_new]
        for n in range(n_layers):
            x = cases[n].forward(batch, x, oracle=False)[0]
        top = torch.from_numpy(np.ascontiguousarray(x[off:off + r.n_new], dtype=np.float32)).to("cuda", dt)
        dwin = torch.empty_like(top)
        B.flexco_lm_loss(head, top, tgt_d[r.start_pos:r.start_pos + r.n_new], r.n_new, 1.0 / L, loss_d, dwin, hws, hb)
        dtop[r.start_pos:r.start_pos + r.n_new] = dwin
        batch = gen.advance(batch, prefill_chunk=prefill_chunk, ft_window=ft_window)
        it += 1
    assert it >= 2

    # ---- backward: layers from the top, each over the windows from the sequence's end -----------------
    pages = batch0.seq_pages[ft_seq]
    pages_d = torch.from_numpy(np.asarray(pages, dtype=np.int32)).to("cuda")
    dcur = dtop
    for n in range(n_layers - 1, -1, -1):
        case = cases[n]
        case.dev.zero_grads()
        case.d_ft[ft_seq].zero_accum()
        dnext = torch.zeros_like(dcur) if n > 0 else None          # nothing trainable below the first layer
        l = L
        for s in bwd_windows:
            print(f"  backward layer {n} window [{l - s}, {l})", flush=True)
            ws = HH.Workspace(case.dev.c, 0, 0, s, l)
            B.flexco_lora_bwd(case.dev.c, case.dev.w, case.dev.lora, case.d_pool.c, pages_d, len(pages), case.d_ft[ft_seq].c,
                              l - s, s, dcur[l - s:l], dnext[l - s:l] if dnext is not None else None, ws.ptr, ws.bytes)
            l -= s
        torch.cuda.synchronize()
        dcur = dnext

    # ---- the definition -------------------------------------------------------------------------------
    loss_o, grads_o, new_loras, new_opt = OT.training_step_whole_seq(cfg, layers, loras, gain, w_lm, x_seq, targets, 1.0 / L,
                                                                     None, 1, lr)
    got_loss = float(loss_d.item())
    print(f"  loss {got_loss:.6f} vs {loss_o:.6f}", flush=True)
    assert abs(got_loss - loss_o) <= tol * abs(loss_o)
    worst = 0.0
    for n in range(n_layers):
        gg = cases[n].dev.grads_numpy()
        assert set(gg) == set(cfg.lora_targets)
        for t in cfg.lora_targets:
            worst = max(worst, assert_close(f"layer {n} dA[{t}]", gg[t][0], grads_o[n][t][0], tol))
            worst = max(worst, assert_close(f"layer {n} dB[{t}]", gg[t][1], grads_o[n][t][1], tol))
    print(f"  worst gradient error {worst:.2e}", flush=True)
    if not adam:
        return
    # ---- Adam on every bypass matrix (fp32 parameters: no master copy) --------------------------------
    for n in range(n_layers):
        dev = cases[n].dev
        for t in cfg.lora_targets:
            for P, G, k in ((dev.A[t], dev.dA[t], 0), (dev.Bm[t], dev.dB[t], 1)):
                m_d, v_d = torch.zeros_like(G), torch.zeros_like(G)
                B.flexco_adam_step(P, None, G, m_d, v_d, P.numel(), HH.DTYPE_CODE[cfg.dtype], lr, 0.9, 0.999, 1e-8, 1)
                torch.cuda.synchronize()
                # a gradient entry within rounding of zero may take its step in either direction: compare
                # where the oracle's gradient is well away from zero, and bound the move everywhere
                go = grads_o[n][t][k]
                new_o, old_o = new_loras[n][t][k], np.asarray(loras[n][t][k], dtype=np.float64)
                got = to_np(P).T
                sure = np.abs(go) > 1e-3 * np.abs(go).max()
                assert sure.mean() > 0.5
                assert np.abs(got - new_o)[sure].max() <= 1e-4 * np.abs(new_o).max(), (n, t, k)
                assert np.abs(got - old_o).max() <= lr * (1 + 1e-5)
                assert_close(f"layer {n} m[{t}]", to_np(m_d).T, new_opt[n][t][2 * k], tol)


def test_training_step_end_to_end_three_layers_f32():
    print("training step, 3 layers, fp32", flush=True)
    b = gen.mixed_batch(16, 11, decode_ctx=(1, 17, 40), prefill=[(0, 5, 40)], finetune=[(0, 24, 64)], extra_capacity=3)
    run_training_step(C1, 3, b, ft_window=24, prefill_chunk=20, bwd_windows=[40, 24], V=203, seed=11, lr=1e-3, adam=True)


def test_training_step_end_to_end_two_layers_bf16():
    print("training step, 2 layers, bf16", flush=True)
    cfg = CONFIGS["c2_llama8b_layer"].with_(name="small_bf16", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408)
    b = gen.batch_scaled(12, 6, 30, 300, [(0, 50, 50)], [(0, 100, 230)])
    run_training_step(cfg, 2, b, ft_window=100, prefill_chunk=32, bwd_windows=[30, 200], V=1000, seed=12, lr=1e-3, adam=False)
