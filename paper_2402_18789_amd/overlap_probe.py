"""Forward of the benchmark batch and the finetune window's backward on two streams (Sec. 6.2: the
backward pass of finetuning runs beside inference): what each costs the other, with the whole chip
shared and with the compute units partitioned between the two streams by CU masks.

    python -m paper_2402_18789_amd.overlap_probe

Prints, per setting, the median duration of the forward call and of the backward call (HIP events on
their own streams) and the wall time of the pair.  The backward window belongs to a finetune sequence
with pages and state of its own, as in bench.py's two-stream run."""
import ctypes as C
import time

import numpy as np
import torch

import paper_2402_18789_amd.binding as B
from paper_2402_18789_amd import host as HH
from workload import gen
from workload.configs import CONFIGS

hip = C.CDLL("libamdhip64.so")


def masked_stream(n_lo, n_hi, total=256):
    """a stream of default priority whose kernels run on the compute units [n_lo, n_hi) only"""
    words = (total + 31) // 32
    arr = (C.c_uint32 * words)()
    for i in range(n_lo, n_hi):
        arr[i // 32] |= (1 << (i % 32))
    st = C.c_void_p()
    rc = hip.hipExtStreamCreateWithCUMask(C.byref(st), C.c_uint32(words), arr)
    assert rc == 0, rc
    return torch.cuda.ExternalStream(st.value)


def main():
    cfg, seed = CONFIGS["c2_llama8b_layer"], 0
    batch = gen.batch_c2(seed)
    W, lora = gen.layer_weights(cfg, seed, 0), gen.lora_weights(cfg, seed, 0)
    layers = [HH.DeviceLayer(cfg, W, lora) for _ in range(3)]
    ft_req = [r for r in batch.requests if r.kind == 2][0]
    n_seq_pages = len(batch.seq_pages[ft_req.seq_id])
    pool = HH.DevicePool(cfg, batch.num_pages + n_seq_pages)
    pool.fill_random(seed)
    L = batch.seq_capacity[ft_req.seq_id]
    ft = HH.DeviceFtState(cfg, L)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    hm = db.host_maps
    T, n_ft = hm.T, hm.n_ft
    ws = HH.Workspace(layers[0].c, T, hm.n_parts, n_ft, L)
    ws_b = HH.Workspace(layers[0].c, T, hm.n_parts, n_ft, L)
    x = torch.from_numpy(gen.layer_input(cfg, seed, T)).to("cuda", torch.bfloat16)
    y = torch.empty_like(x)
    dY = torch.from_numpy(gen.layer_input(cfg, seed, n_ft, tag="dy")).to("cuda", torch.bfloat16)
    dX = torch.empty_like(dY)
    ft_pages = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")
    ly = layers[0]
    B.flexco_layer_forward(ly.c, ly.w, ly.lora, db.maps, x, y, pool.c, ft.c, ws.ptr, ws.bytes)
    torch.cuda.synchronize()
    bwd_pages = torch.arange(batch.num_pages, batch.num_pages + n_seq_pages, device="cuda")
    pool.k[bwd_pages] = pool.k[ft_pages.long()]
    pool.v[bwd_pages] = pool.v[ft_pages.long()]
    ft_b = HH.DeviceFtState(cfg, L)
    for name in ("q_cache", "attn", "x", "x2", "gate", "up", "lse"):
        getattr(ft_b, name).copy_(getattr(ft, name))
    for t in ft_b.u:
        ft_b.u[t].copy_(ft.u[t])
    bwd_pages = bwd_pages.to(torch.int32)
    torch.cuda.synchronize()
    def run(sa, sb, do_f=True, do_b=True, iters=20):
        tf, tb, tw = [], [], []
        for i in range(iters + 3):
            ly = layers[i % 3]
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if do_f:
                e[0].record(sa)
                B.flexco_layer_forward(ly.c, ly.w, ly.lora, db.maps, x, y, pool.c, ft.c, ws.ptr, ws.bytes, stream=sa)
                e[1].record(sa)
            if do_b:
                e[2].record(sb)
                B.flexco_lora_bwd(ly.c, ly.w, ly.lora, pool.c, bwd_pages, n_seq_pages, ft_b.c, ft_req.start_pos,
                                  ft_req.n_new, dY, dX, ws_b.ptr, ws_b.bytes, stream=sb)
                e[3].record(sb)
            torch.cuda.synchronize()
            if i >= 3:
                tw.append((time.perf_counter() - t0) * 1e3)
                if do_f:
                    tf.append(e[0].elapsed_time(e[1]))
                if do_b:
                    tb.append(e[2].elapsed_time(e[3]))
        med = lambda v: float(np.median(v)) if v else float("nan")
        return med(tf), med(tb), med(tw)
    s0, s1 = torch.cuda.Stream(), torch.cuda.Stream()
    print("forward alone        : fwd %.3f ms" % run(s0, s1, True, False)[0], flush=True)
    print("backward alone       : bwd %.3f ms" % run(s0, s1, False, True)[1], flush=True)
    f, b, w = run(s0, s1)
    print("both, no masks       : fwd %.3f  bwd %.3f  wall %.3f" % (f, b, w), flush=True)
    for n in (32, 64, 96, 128):
        sa, sb = masked_stream(0, 256 - n), masked_stream(256 - n, 256)
        fa = run(sa, sb, True, False)[0]
        ba = run(sa, sb, False, True)[1]
        f, b, w = run(sa, sb)
        print("bwd on %3d CUs, fwd on the other %3d : alone fwd %.3f bwd %.3f | both fwd %.3f  bwd %.3f  wall %.3f"
              % (n, 256 - n, fa, ba, f, b, w), flush=True)


if __name__ == "__main__":
    main()
