"""The layer calls under HIP graph capture.  The library allocates nothing, never synchronises and records
no memset or copy nodes, so one co-serving iteration can be captured once and replayed (the way a serving
loop removes the host's launch cost for small batches).  Every replay is checked bit for bit against the
eager run, with eager work and synchronisations of the program's own between the replays."""
import numpy as np
import pytest
import torch

import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH
from workload import gen
from workload.configs import CONFIGS, KIND_FINETUNE

pytestmark = pytest.mark.gpu

C2 = CONFIGS["c2_llama8b_layer"]
SMALL_BF16 = C2.with_(name="small_bf16", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408)


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("chunk_path", [-1, 2])
def test_layer_forward_and_window_backward_replay_from_a_graph(chunk_path):
    """chunk_path 2: the attention's chunk items run on the library's side stream, which leaves the captured stream and
    rejoins it inside the call (flexco_attention_chunk_path); the eager run before the capture has created it."""
    B.flexco_attention_chunk_path(chunk_path)
    try:
        _replay_from_a_graph(chunk_path)
    finally:
        B.flexco_attention_chunk_path(-1)


def _replay_from_a_graph(chunk_path):
    cfg, seed = SMALL_BF16, 5
    say(f"graph capture: mixed batch forward + window backward, chunk_path={chunk_path}")
    batch = gen.batch_scaled(seed, 9, 3, 400, [(0, 70, 70), (128, 64, 300)], [(96, 64, 160)])
    W, lora = gen.layer_weights(cfg, seed, 0), gen.lora_weights(cfg, seed, 0)
    dev = HH.DeviceLayer(cfg, W, lora)
    pool = HH.DevicePool(cfg, batch.num_pages)
    pool.fill_random(seed)
    ft_req = [r for r in batch.requests if r.kind == KIND_FINETUNE][0]
    L = batch.seq_capacity[ft_req.seq_id]
    ft = HH.DeviceFtState(cfg, L)
    # rows before the window: what earlier iterations would have left (any finite values serve)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    for name in ("q_cache", "x", "x2", "gate", "up", "attn"):
        t = getattr(ft, name)
        t.copy_(torch.randn(t.shape, generator=g, device="cuda", dtype=torch.float32).to(t.dtype))
    ft.lse.fill_(3.0)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    T = db.host_maps.T
    ws = HH.Workspace(dev.c, T, db.host_maps.n_parts, ft_req.n_new, ft_req.start_pos + ft_req.n_new)
    x = torch.from_numpy(gen.layer_input(cfg, seed, T)).to("cuda", torch.bfloat16)
    y = torch.empty_like(x)
    dY = torch.from_numpy(gen.layer_input(cfg, seed, ft_req.n_new, tag="dy")).to("cuda", torch.bfloat16)
    dX = torch.empty_like(dY)
    pages_d = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")

    def step():
        B.flexco_layer_forward(dev.c, dev.w, dev.lora, db.maps, x, y, pool.c, ft.c, ws.ptr, ws.bytes)
        B.flexco_lora_bwd(dev.c, dev.w, dev.lora, pool.c, pages_d, int(pages_d.numel()), ft.c, ft_req.start_pos,
                          ft_req.n_new, dY, dX, ws.ptr, ws.bytes)

    def results():
        torch.cuda.synchronize()
        out = [y.clone(), dX.clone(), ft.dk_accum.clone(), ft.dv_accum.clone()]
        out += [dev.dA[t].clone() for t in dev.dA] + [dev.dB[t].clone() for t in dev.dB]
        return out

    def reset():
        dev.zero_grads()
        ft.zero_accum()
        y.zero_()
        dX.zero_()

    reset()
    step()
    eager = results()
    assert all(torch.isfinite(t.float()).all() for t in eager)

    graph = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    say("  capture")
    with torch.cuda.graph(graph):
        step()
    for i in range(3):
        say(f"  replay {i}")
        reset()                                   # eager work between the replays
        x.add_(0.0)
        torch.cuda.synchronize()
        graph.replay()
        got = results()
        for a, b in zip(got, eager):
            assert torch.equal(a, b), f"replay {i} differs from the eager run"
    # a replay reads its inputs where they lie: new input rows, same graph
    x2 = torch.from_numpy(gen.layer_input(cfg, seed + 1, T)).to("cuda", torch.bfloat16)
    x.copy_(x2)
    reset()
    step()
    eager2 = results()
    reset()
    graph.replay()
    for a, b in zip(results(), eager2):
        assert torch.equal(a, b), "replay on new inputs differs from the eager run"
    assert not torch.equal(eager2[0], eager[0])
