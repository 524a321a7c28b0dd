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
    for i in ignore:
        y[i] = -1
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
