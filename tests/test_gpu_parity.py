"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X).

Bar: index maps bit-exact (tests/test_abi_host.py); outputs and LoRA gradients within
1e-4 (fp32 tiny configuration) or 2e-2 (bf16) max relative error per tensor,
max|gpu - oracle| / max|oracle|.
"""
import numpy as np
import pytest
import torch

from workload import gen, CONFIGS
from workload.configs import KIND_FINETUNE

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from oracle import ops as OO, layer as OL
    from oracle.maps import build_maps
    from gpu_common import Case, rel_err, elem_err, to_np, TOL, assert_close, assert_close_storage

C1 = CONFIGS["c1_tiny_f32"]
C2 = CONFIGS["c2_llama8b_layer"]
# bf16 shapes small enough for the oracle in seconds, still several tiles and ragged tails
SMALL_BF16 = C2.with_(name="small_bf16", hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=1408)
SMALL_BF16_G5 = C2.with_(name="small_bf16_g5", hidden=640, n_q_heads=10, n_kv_heads=2, head_dim=128, ffn=1152,
                         lora_targets=("q", "k", "v", "o", "gate", "up", "down"), qkv_bias=True, rms_eps=1e-6,
                         rope_theta=1e6)


# kv groups of one (every query head has its own kv head) and of eight query heads
SMALL_BF16_MHA = C2.with_(name="small_bf16_mha", hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128, ffn=1408)
SMALL_BF16_G8 = C2.with_(name="small_bf16_g8", hidden=1024, n_q_heads=8, n_kv_heads=1, head_dim=128, ffn=1408)


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------------
# dense projection
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,K,trans", [(68, 768, 256, 0), (68, 256, 688, 0), (33, 100, 72, 1), (256, 512, 1024, 0),
                                         (1024, 1536, 512, 0), (300, 1408, 512, 1), (256, 4096, 1024, 1),
                                         (1, 256, 256, 0), (129, 384, 136, 0),
                                         # a single k-stage (the bottleneck adapter's two projections)
                                         (200, 512, 64, 0), (130, 640, 64, 1),
                                         # >= 192 tiles of 256 x 256: the large-tile kernel, ragged in M and N,
                                         # odd and even numbers of k-stages
                                         (300, 49160, 320, 0), (520, 24584, 192, 0), (256, 49152, 64, 0),
                                         # 192-wide tiles (one round of 128 x 192), ragged in N; 256-wide and
                                         # 192-wide tiles side by side in one product
                                         (1024, 6152, 128, 0), (1024, 28672, 64, 0), (1000, 28680, 128, 0),
                                         # more 128 x 128 tiles than CUs (450): the two-stage blocks that share a CU, ragged in
                                         # M and N, odd number of k-stages
                                         (1100, 6344, 320, 0),
                                         # input-gradient form on 256 x 256 tiles (a window of 512 rows or more whose
                                         # large tiles fill most of the CUs in one round), ragged in M and N, odd and
                                         # even numbers of k-stages
                                         (1000, 13832, 320, 1), (700, 18184, 128, 1)])
def test_gemm(dtype, M, N, K, trans):
    say(f"gemm {dtype} M={M} N={N} K={K} trans={trans}")
    cfg = C1.with_(dtype=dtype)
    g = gen.rng(5, "gemm", M, N, K, trans)
    A = gen.storage_round(cfg, g.standard_normal((M, K), dtype=np.float32))
    W = gen.storage_round(cfg, g.standard_normal((K, N) if trans else (N, K), dtype=np.float32))
    bias = gen.storage_round(cfg, g.standard_normal(N, dtype=np.float32))
    res = gen.storage_round(cfg, g.standard_normal((M, N), dtype=np.float32))
    dt = HH.TORCH_DTYPE[dtype]
    dev = lambda a: torch.from_numpy(a).to("cuda", dt)
    A_d, W_d, b_d, r_d = dev(A), dev(W), dev(bias), dev(res)
    C_d = torch.empty((M, N), dtype=dt, device="cuda")
    A64, W64 = A.astype(np.float64), W.astype(np.float64)
    ref = A64 @ (W64 if trans else W64.T)
    B.flexco_gemm(A_d, W_d, C_d, None, None, M, N, K, trans, HH.DTYPE_CODE[dtype])
    torch.cuda.synchronize()
    assert_close("gemm", to_np(C_d), ref, TOL[dtype])
    if not trans:
        B.flexco_gemm(A_d, W_d, C_d, b_d, r_d, M, N, K, trans, HH.DTYPE_CODE[dtype])
        torch.cuda.synchronize()
        assert_close("gemm+bias+res", to_np(C_d), ref + bias + res, TOL[dtype])


# ------------------------------------------------------------------------------------------
# segmented LoRA forward
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,din,dout,r", [("f32", 256, 688, 8), ("bf16", 512, 1408, 16), ("bf16", 1408, 512, 32),
                                              ("f32", 72, 40, 3)])
def test_lora_fwd_segments(dtype, din, dout, r):
    say(f"lora_fwd {dtype} in={din} out={dout} r={r}")
    cfg = C1.with_(dtype=dtype)
    T = 77
    seg_off, seg_adapter = [0, 9, 30, 31, 60, 77], [-1, 1, 0, -1, 1]
    g = gen.rng(6, "lora", din, dout, r)
    rnd = lambda shape, s=1.0: gen.storage_round(cfg, (g.standard_normal(shape) * s).astype(np.float32))
    x, y0 = rnd((T, din)), rnd((T, dout))
    As = [rnd((din, r), 0.05) for _ in range(2)]
    Bs = [rnd((r, dout), 0.05) for _ in range(2)]
    dt = HH.TORCH_DTYPE[dtype]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dt)
    x_d, y_d = dev(x), dev(y0)
    A_d, B_d = [dev(a.T) for a in As], [dev(b.T) for b in Bs]
    u = torch.zeros(T * r, dtype=torch.float32, device="cuda")
    B.flexco_lora_fwd(x_d, y_d, T, din, dout, r, 2.0, HH.DTYPE_CODE[dtype], A_d, B_d, seg_off, seg_adapter, u)
    torch.cuda.synchronize()
    ref = y0.astype(np.float64)
    for s, a in enumerate(seg_adapter):
        if a >= 0:
            rows = slice(seg_off[s], seg_off[s + 1])
            ref[rows] += OO.lora_delta(x[rows].astype(np.float64), As[a].astype(np.float64), Bs[a].astype(np.float64), 2.0)
    got = to_np(y_d)
    assert_close("lora_fwd", got, ref, TOL[dtype])
    for s, a in enumerate(seg_adapter):          # rows without adapter are untouched, bit for bit
        if a < 0:
            assert np.array_equal(got[seg_off[s]:seg_off[s + 1]], y0[seg_off[s]:seg_off[s + 1]].astype(np.float64))


# ------------------------------------------------------------------------------------------
# mixed attention alone
# ------------------------------------------------------------------------------------------
def attention_case(cfg, batch, split, seed=3):
    case = Case(cfg, batch, seed=seed, kv_split_pages=split)
    om = build_maps(batch.requests, batch.seq_pages, batch.page_size, batch.num_pages)
    T = om["T"]
    g = gen.rng(seed, "attnq", cfg.name, T)
    q = gen.storage_round(cfg, g.standard_normal((T, cfg.q_dim), dtype=np.float32))
    # K/V of the batch's own tokens, seeded, on both sides
    for r in batch.requests:
        k, v = gen.kv_prefix(cfg, seed + 1, 0, r.seq_id, r.start_pos + r.n_new)
        pages = batch.seq_pages[r.seq_id]
        sl = case.o_pool.slots(pages, r.start_pos + r.n_new)[r.start_pos:]
        case.o_pool.k[sl], case.o_pool.v[sl] = k[r.start_pos:], v[r.start_pos:]
        case.d_pool.write_rows(pages, k[r.start_pos:], v[r.start_pos:], start=r.start_pos)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages, split)
    ws = HH.Workspace(case.dev.c, T, db.host_maps.n_parts)
    dt = HH.TORCH_DTYPE[cfg.dtype]
    q_d = torch.from_numpy(q).to("cuda", dt)
    out_d = torch.empty_like(q_d)
    lse_d = torch.empty((T, cfg.n_q_heads), dtype=torch.float32, device="cuda")
    B.flexco_attention_mixed(case.dev.c, db.maps, q_d, case.d_pool.c, out_d, lse_d, ws.ptr, ws.bytes)
    torch.cuda.synchronize()
    a_o, lse_o = OL.attention_mixed(cfg, om, q.astype(np.float64), case.o_pool)
    return to_np(out_d), a_o, to_np(lse_d), lse_o


# chunk_path: which kernel takes the prefill chunks and finetune windows (flexco_attention_chunk_path): 0 = the one that
# streams the decode tokens, 1 = the four-wavefront kernel with K / V staged in LDS
@pytest.mark.parametrize("chunk_path", [0, 1, 2])
@pytest.mark.parametrize("name,split", [("c1", 0), ("c1", 2), ("small_bf16", 0), ("small_bf16", 2), ("g5", 4), ("mha", 2),
                                        ("g8", 4), ("long", 0), ("small_bf16", 6), ("long", 250), ("windows", 0), ("windows", 32)])
def test_attention_mixed(name, split, chunk_path):
    say(f"attention_mixed {name} split={split} chunk_path={chunk_path}")
    B.flexco_attention_chunk_path(chunk_path)
    try:
        _attention_mixed(name, split)
    finally:
        B.flexco_attention_chunk_path(-1)


def _attention_mixed(name, split):
    if name == "c1":
        cfg, batch = C1, gen.batch_c1(0)
    elif name == "small_bf16":
        cfg = SMALL_BF16
        batch = gen.batch_scaled(4, 12, 1, 700, [(0, 150, 150), (200, 77, 300)], [(96, 75, 171)])
    elif name == "g5":
        cfg = SMALL_BF16_G5
        batch = gen.batch_scaled(5, 7, 17, 333, [(0, 40, 40)], [(64, 100, 164)])
    elif name == "long":                     # the longest contexts of the larger configurations: 16 key splits
        cfg = SMALL_BF16
        batch = gen.mixed_batch(16, 8, decode_ctx=(16384, 8191, 4097, 1), prefill=[(7000, 100, 7100)],
                                finetune=[(3840, 256, 4096)])
    elif name == "windows":                  # no decode token at all (by default the four-wavefront kernel's case): a prompt
        cfg = SMALL_BF16_G5                  # from position 0 and a window on a long prefix, 113 pages (an odd number of stages)
        batch = gen.mixed_batch(16, 0, decode_ctx=(), prefill=[(0, 300, 300)], finetune=[(1500, 300, 1800)])
    elif name == "mha":
        cfg = SMALL_BF16_MHA                 # 16 tokens per tile, 64 per work item
        batch = gen.batch_scaled(6, 5, 9, 200, [(0, 150, 150), (40, 77, 117)], [(30, 100, 130)])
    else:
        cfg = SMALL_BF16_G8                  # 2 tokens per tile
        batch = gen.batch_scaled(7, 6, 20, 260, [(0, 45, 45)], [(64, 37, 101)])
    out, a_o, lse, lse_o = attention_case(cfg, batch, split)
    assert_close("attention out", out, a_o, TOL[cfg.dtype])
    assert float(np.max(np.abs(lse - lse_o))) <= (1e-4 if cfg.dtype == "f32" else 2e-2)


# ------------------------------------------------------------------------------------------
# attention backward of one token window alone (Sec. 6.1): dQ of the window, dK/dV accumulated
# into every cached row before the window's end
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_name,win_start,win_len", [
    ("small_bf16", 0, 40),          # the first window: every row sees only the window itself, ragged page
    ("small_bf16", 96, 75),         # ragged start and end, l = 171 (not a multiple of 16)
    ("small_bf16", 448, 64),        # aligned, several key blocks of 64 before the window
    ("small_bf16", 301, 131),       # window longer than a row block, odd everything
    ("g5", 130, 33),                # kv group of 5 query heads
    ("mha", 70, 90),                # kv group of 1: the second half of a dK/dV block has no head of its own
    ("g8", 17, 50),                 # kv group of 8
    ("c1", 5, 6),                   # fp32 generic path
    ("small_bf16", 3840, 256),      # the last window of a 4096-token sequence
    ("small_bf16", 8000, 192),      # of an 8192-token one
    ("c2", 203, 530),               # 17 row blocks x 32 heads: the grid of two blocks per CU (dQ kernel with four pages per
                                    # step), 46 pages (not a multiple of 4), ragged start and end
    ("c2", 2100, 77),               # 35 key blocks x 8 kv heads: more dK/dV blocks than CUs (four-wavefront blocks)
])
def test_attention_window_bwd(cfg_name, win_start, win_len):
    say(f"attention_window_bwd {cfg_name} window [{win_start}, +{win_len})")
    cfg = {"small_bf16": SMALL_BF16, "g5": SMALL_BF16_G5, "mha": SMALL_BF16_MHA, "g8": SMALL_BF16_G8, "c1": C1, "c2": C2}[cfg_name]
    l = win_start + win_len
    ps = cfg.page_size
    n_pages = (l + ps - 1) // ps
    g = gen.rng(11, "attnbwd", cfg.name, win_start, win_len)
    pages = (g.permutation(n_pages + 3)[:n_pages] + 1).astype(np.int32)      # scattered, page 0 unused
    k_rows, v_rows = gen.kv_prefix(cfg, 12, 0, 0, l)
    q = gen.storage_round(cfg, g.standard_normal((win_len, cfg.q_dim), dtype=np.float32)).astype(np.float64)
    dout = gen.storage_round(cfg, g.standard_normal((win_len, cfg.q_dim), dtype=np.float32)).astype(np.float64)
    q_pos = np.arange(win_start, l)
    kk, vv = k_rows.astype(np.float64), v_rows.astype(np.float64)
    out_o, lse_o = OO.attention(q, q_pos, kk, vv, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    dq_o, dk_o, dv_o = OO.attention_bwd(q, q_pos, kk, vv, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dout)

    dcfg = HH.c_cfg(cfg)
    pool = HH.DevicePool(cfg, n_pages + 4)
    pool.fill_random(5)                     # slots that are never written hold arbitrary finite values
    pool.write_rows(pages, k_rows, v_rows)
    dt = HH.TORCH_DTYPE[cfg.dtype]
    dev = lambda a, d=dt: torch.from_numpy(np.ascontiguousarray(a)).to("cuda", d)
    q_d, out_d, dout_d = dev(q), dev(gen.storage_round(cfg, out_o.astype(np.float32))), dev(dout)
    lse_d = dev(lse_o, torch.float32)
    dq_d = torch.empty_like(q_d)
    # accumulators start from a seeded non-zero state: the call must add, not overwrite
    base_k = g.standard_normal((l + 3, cfg.kv_dim), dtype=np.float32)
    base_v = g.standard_normal((l + 3, cfg.kv_dim), dtype=np.float32)
    dk_d, dv_d = dev(base_k, torch.float32), dev(base_v, torch.float32)
    ws = torch.empty(win_len * cfg.n_q_heads * 4 + 1024, dtype=torch.uint8, device="cuda")
    pages_d = torch.from_numpy(pages).to("cuda")
    B.flexco_attention_window_bwd(dcfg, pool.c, pages_d, n_pages, win_start, win_len, q_d, out_d, lse_d, dout_d, dq_d,
                                  dk_d, dv_d, ws, ws.numel())
    torch.cuda.synchronize()
    tol = TOL[cfg.dtype]
    assert_close("dq", to_np(dq_d), dq_o, tol)
    assert_close("dk_accum", to_np(dk_d)[:l] - base_k[:l], dk_o, tol)
    assert_close("dv_accum", to_np(dv_d)[:l] - base_v[:l], dv_o, tol)
    assert np.array_equal(to_np(dk_d)[l:], base_k[l:].astype(np.float64))   # rows past the window's end untouched
    assert np.array_equal(to_np(dv_d)[l:], base_v[l:].astype(np.float64))


# ------------------------------------------------------------------------------------------
# whole layer: forward iterations, then token-window backward
# ------------------------------------------------------------------------------------------
def run_layer_case(cfg, batch0, ft_window, prefill_chunk, bwd_windows, seed=0, split=0, need_dx=True,
                   keep_u=True, adapters=None, ft_adapter=0, gpu_page_shift=0, storage_exceptions=()):
    """Forward iterations until the finetune sequence is through, then its token-window backward, both sides in
    lock step; every output, saved activation, accumulator and LoRA gradient held to the plain oracle at the
    configuration's bar.  storage_exceptions: names of the tensors of THIS case that may miss the 2e-2 bf16 bar
    against the plain oracle under the rule of assert_close_storage (the device is no further out than 1.5 times
    what exact arithmetic with bf16 storage is); any other tensor missing the bar fails."""
    report, excess = [], []
    tol = TOL[cfg.dtype]
    case = Case(cfg, batch0, seed=seed, kv_split_pages=split, keep_u=keep_u, adapters=adapters, gpu_page_shift=gpu_page_shift,
                lora=adapters[ft_adapter] if adapters is not None else None, storage_oracle=True)
    bf16 = case.storage is not None

    def check(name, got, ref, ref_s):
        e, es = assert_close_storage(name, got, ref, ref_s if bf16 else None, tol, report)
        if e > tol:
            excess.append(name)
        return e

    batch, it = batch0, 0
    ft_seq = [r.seq_id for r in batch0.requests if r.kind == KIND_FINETUNE][0]
    L = batch0.seq_capacity[ft_seq]
    y_ft_g, y_ft_o = np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden))
    while any(r.kind == KIND_FINETUNE for r in batch.requests):
        say(f"  forward iteration {it}: T={batch.n_tokens}")
        x = gen.layer_input(cfg, seed, batch.n_tokens, tag=f"x{it}")
        y_g, y_o, db = case.forward(batch, x)
        check(f"y it{it}", y_g, y_o, case.last_y_s)
        for r, off in zip(batch.requests, np.cumsum([0] + [q.n_new for q in batch.requests])):
            kg, vg = case.d_pool.read_rows(case.dpages(batch.seq_pages[r.seq_id]), r.n_new, r.start_pos)
            sl = case.o_pool.slots(batch.seq_pages[r.seq_id], r.start_pos + r.n_new)[r.start_pos:]
            assert_close(f"K append it{it}", kg, case.o_pool.k[sl], tol)
            assert_close(f"V append it{it}", vg, case.o_pool.v[sl], tol)
            if r.kind == KIND_FINETUNE:
                y_ft_g[r.start_pos:r.start_pos + r.n_new] = y_g[off:off + r.n_new]
                y_ft_o[r.start_pos:r.start_pos + r.n_new] = y_o[off:off + r.n_new]
        batch = gen.advance(batch, prefill_chunk=prefill_chunk, ft_window=ft_window)
        it += 1
    st_d, st_o = case.d_ft[ft_seq], case.o_ft[ft_seq]
    st_s = case.s_ft.get(ft_seq)
    for name in ("q_cache", "x", "x2", "gate", "up", "attn", "lse"):
        check("saved " + name, to_np(getattr(st_d, name)), getattr(st_o, name), getattr(st_s, name) if bf16 else None)
    # backward: loss = MSE to seeded targets on the finetune sequence's layer output (oracle's dY on
    # both sides, so that the backward pass is compared on identical inputs)
    target = gen.loss_targets(cfg, seed, L).astype(np.float64)
    _, dY = OL.mse_loss_grad(y_ft_o, target)
    dY = gen.storage_round(cfg, (dY * L * cfg.hidden).astype(np.float32)).astype(np.float64)   # O(1) magnitudes
    grads_o = {}
    case.dev.zero_grads()
    st_d.zero_accum()
    l = L
    dX_g, dX_o, dX_s = np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden))
    for s in bwd_windows:
        say(f"  backward window [{l - s}, {l})")
        g, o = case.backward_window(ft_seq, l - s, s, dY[l - s:l], grads_o, need_dx)
        if need_dx:
            dX_g[l - s:l], dX_o[l - s:l] = g, o
            if bf16:
                dX_s[l - s:l] = case.last_dx_s
        l -= s
    assert l == 0
    if need_dx:
        check("dX", dX_g, dX_o, dX_s)
    check("dk_accum", to_np(st_d.dk_accum), st_o.dk_accum, st_s.dk_accum if bf16 else None)
    check("dv_accum", to_np(st_d.dv_accum), st_o.dv_accum, st_s.dv_accum if bf16 else None)
    grads_g = case.dev.grads_numpy()
    assert set(grads_g) == set(grads_o) == set(cfg.lora_targets)
    for t in cfg.lora_targets:
        check(f"dA[{t}]", grads_g[t][0], grads_o[t][0], case.grads_s[t][0] if bf16 else None)
        check(f"dB[{t}]", grads_g[t][1], grads_o[t][1], case.grads_s[t][1] if bf16 else None)
    # per tensor: device vs plain oracle (and, bf16: what bf16 storage with exact arithmetic alone costs)
    say("  " + ", ".join(f"{r[0]}={r[1]:.1e}" + (f"({r[2]:.1e})" if len(r) > 2 else "") for r in report))
    unexpected = [n for n in excess if n not in storage_exceptions]
    assert not unexpected, "tensors beyond %.0e against the plain oracle that this case does not list as storage-" \
                           "rounding exceptions: %s" % (tol, unexpected)
    case.excess = excess
    return case, report


def test_layer_c1_two_iterations_and_backward():
    say("layer c1")
    run_layer_case(C1, gen.batch_c1(0), ft_window=32, prefill_chunk=32, bwd_windows=[32, 32])


def test_layer_c1_uneven_windows_and_split_keys():
    say("layer c1 uneven")
    b = gen.mixed_batch(16, 1, decode_ctx=(1, 17, 64), prefill=[(0, 5, 40)], finetune=[(0, 23, 64)], extra_capacity=3)
    run_layer_case(C1, b, ft_window=41, prefill_chunk=35, bwd_windows=[1, 40, 23], split=2)


def test_layer_c1_no_input_grad_all_targets():
    say("layer c1 all targets, dX = NULL")
    cfg = C1.with_(lora_targets=("q", "k", "v", "o", "gate", "up", "down"), qkv_bias=True)
    run_layer_case(cfg, gen.batch_c1(2), ft_window=32, prefill_chunk=32, bwd_windows=[64], need_dx=False)


def test_layer_c1_down_only():
    say("layer c1 down-only LoRA")
    cfg = C1.with_(lora_targets=("down",))
    run_layer_case(cfg, gen.batch_c1(3), ft_window=32, prefill_chunk=32, bwd_windows=[20, 44])


def test_layer_small_bf16():
    say("layer small bf16")
    b = gen.batch_scaled(7, 10, 3, 600, [(0, 130, 130), (256, 64, 400)], [(0, 100, 260)])
    run_layer_case(SMALL_BF16, b, ft_window=160, prefill_chunk=70, bwd_windows=[60, 200], seed=7)


@pytest.mark.parametrize("rank", [8, 24, 48, 64])
def test_layer_small_bf16_other_ranks(rank):
    """LoRA ranks other than the configurations' 16 and 32, on all seven projections: 48 and 64 take the
    matrix-core LoRA kernels with three and four rank tiles, 8 and 24 the type-generic ones.  Backward windows of
    300 rows: the gradient launch walks more than one 256-row chunk."""
    say("layer small bf16, LoRA rank %d" % rank)
    cfg = SMALL_BF16_G5.with_(name="small_bf16_r%d" % rank, lora_rank=rank)
    b = gen.batch_scaled(11, 6, 3, 300, [(0, 90, 90)], [(0, 300, 600)])
    run_layer_case(cfg, b, ft_window=300, prefill_chunk=90, bwd_windows=[300, 300], seed=11)


def test_layer_bf16_head_dim_64_runs_on_the_generic_attention_kernels_and_says_so():
    """bf16 with head_dim 64: outside the matrix-core attention kernels' shapes; the layer still meets the bf16 bar
    (type-generic attention kernels, matrix-core projections) and the library counts the fallback."""
    say("layer bf16 head_dim 64 (generic attention kernels)")
    cfg = C2.with_(name="small_bf16_d64", hidden=512, n_q_heads=8, n_kv_heads=4, head_dim=64, ffn=1408)
    b = gen.batch_scaled(12, 7, 3, 300, [(0, 70, 70), (64, 40, 200)], [(0, 60, 150)])
    B.flexco_bf16_fallbacks(reset=True)
    run_layer_case(cfg, b, ft_window=90, prefill_chunk=50, bwd_windows=[50, 100], seed=12)
    n = B.flexco_bf16_fallbacks(reset=True)
    say("  fallbacks: %s" % n)
    assert n["attn_fwd"] > 0 and n["attn_bwd"] > 0 and n["gemm_fwd"] == 0 and n["gemm_bwd"] == 0
    run_layer_case(SMALL_BF16, gen.batch_scaled(7, 10, 3, 600, [(0, 130, 130)], [(0, 100, 100)]), ft_window=100, prefill_chunk=70,
                   bwd_windows=[100], seed=7)
    n = B.flexco_bf16_fallbacks()
    assert all(v == 0 for v in n.values()), n          # head_dim 128: everything on the matrix-core kernels


def test_layer_small_bf16_pool_astride_4gib():
    """A paged pool larger than 2^31 elements (4 GiB) per K and V: the batch's pages sit on both sides of
    that offset, so every kernel that addresses the pool (append, attention forward, its backward) needs
    64-bit offsets."""
    say("layer small bf16, pages astride the 4 GiB offset of the pool")
    cfg = SMALL_BF16
    b = gen.batch_scaled(9, 8, 3, 500, [(0, 100, 100), (128, 64, 300)], [(0, 96, 224)])
    page_elems = cfg.n_kv_heads * cfg.page_size * cfg.head_dim
    boundary_page = (1 << 31) // page_elems
    shift = boundary_page - b.num_pages // 2
    case, _ = run_layer_case(cfg, b, ft_window=128, prefill_chunk=70, bwd_windows=[100, 124], seed=9, gpu_page_shift=shift)
    used = np.concatenate([case.dpages(p) for p in b.seq_pages.values()])
    assert used.min() < boundary_page <= used.max()


def test_layer_small_bf16_group5_all_targets():
    say("layer small bf16 group 5")
    b = gen.batch_scaled(8, 6, 30, 200, [(0, 50, 50)], [(0, 90, 170)])
    run_layer_case(SMALL_BF16_G5, b, ft_window=80, prefill_chunk=16, bwd_windows=[170], seed=8, split=4)


def test_layer_small_bf16_without_kept_rank_products():
    """The state does not keep x A^T of the forward pass: the backward pass multiplies again."""
    say("layer small bf16, saved_u = NULL")
    b = gen.batch_scaled(9, 5, 3, 300, [(0, 40, 40)], [(0, 100, 260)])
    run_layer_case(SMALL_BF16, b, ft_window=160, prefill_chunk=70, bwd_windows=[60, 200], seed=9, keep_u=False)


# Several adapters served in one batch (Sec. 6.2): decode and prefill requests under adapters 1, 2, 3 and
# under none, the finetune sequence under the adapter being trained; then that adapter's backward pass.
@pytest.mark.parametrize("name,n_adapters,ft_adapter", [("c1", 3, 0), ("small_bf16", 4, 2), ("small_bf16", 6, 0)])
def test_layer_with_several_adapters_in_one_batch(name, n_adapters, ft_adapter):
    say(f"layer {name}, {n_adapters} adapters in one batch, finetune on adapter {ft_adapter}")
    if name == "c1":
        cfg = C1
        b = gen.mixed_batch(16, 21, decode_ctx=(16, 32, 48, 64, 7, 20), prefill=[(0, 32, 64), (5, 20, 40)],
                            finetune=[(0, 32, 64)], extra_capacity=2, ft_adapter=ft_adapter)
        kw = dict(ft_window=32, prefill_chunk=32, bwd_windows=[40, 24])
    else:
        cfg = SMALL_BF16
        b = gen.mixed_batch(16, 22, decode_ctx=tuple(range(30, 400, 37)), prefill=[(0, 130, 130), (256, 64, 400)],
                            finetune=[(0, 100, 260)], extra_capacity=3, ft_adapter=ft_adapter)
        kw = dict(ft_window=160, prefill_chunk=70, bwd_windows=[60, 200])
    ids = [-1] + [a for a in range(n_adapters)]                    # inference requests cycle through none, 0, 1, ...
    b = gen.with_adapters(b, ids)
    adapters = [gen.lora_weights(cfg, 23, 0, adapter=a, b_std=0.02) for a in range(n_adapters)]
    run_layer_case(cfg, b, seed=23, adapters=adapters, ft_adapter=ft_adapter, **kw)


def test_several_adapters_error_paths():
    cfg = C1
    b = gen.with_adapters(gen.batch_c1(0), [2, -1])              # adapter id 2 is used
    case = Case(cfg, b, seed=1)
    db = HH.DeviceBatch(cfg, b.requests, b.seq_pages, b.num_pages)
    assert db.host_maps.n_adapters == 3 and db.host_maps.ft_adapter == 0
    ws = HH.Workspace(case.dev.c, db.host_maps.T, db.host_maps.n_parts)
    x = torch.zeros((db.host_maps.T, cfg.hidden), device="cuda")
    y = torch.empty_like(x)
    ft = case.d_ft[[r.seq_id for r in b.requests if r.kind == KIND_FINETUNE][0]].c
    with pytest.raises(B.FlexcoError):                            # two adapters given, id 2 asked for
        B.flexco_layer_forward_multi(case.dev.c, case.dev.w, [case.dev.lora, case.dev.lora], db.maps, x, y, case.d_pool.c, ft,
                                     ws.ptr, ws.bytes)
    with pytest.raises(B.FlexcoError):                            # adapter 2 has a NULL matrix
        B.flexco_layer_forward_multi(case.dev.c, case.dev.w, [case.dev.lora, case.dev.lora, B.Lora()], db.maps, x, y,
                                     case.d_pool.c, ft, ws.ptr, ws.bytes)
    # adapter 1 has no tokens in this batch: it is not looked at
    B.flexco_layer_forward_multi(case.dev.c, case.dev.w, [case.dev.lora, B.Lora(), case.dev.lora], db.maps, x, y, case.d_pool.c,
                                 ft, ws.ptr, ws.bytes)
    torch.cuda.synchronize()


# The 14B / 32B shapes on short sequences (<= 96 keys).  Outputs, saved activations and every gradient that
# does not pass through the softmax logits meet the 2e-2 bar.  The gradients through the logits (dX, the K
# accumulator, dA / dB of q and k) do not, and cannot with this storage type: the oracle run with exact fp64
# arithmetic and bf16 STORAGE (cached q / k / v rows, saved activations, every gradient handed from one operator
# to the next) is itself 2.1e-2 .. 3.2e-2 away from the unrounded oracle on exactly these tensors (one rounded
# element of a cached key moves that key's logit for every query of the group; 64 .. 96 keys do not average that
# away as the 2048 .. 4096 keys of the full-size cases do, where the same tensors stay below 1.2e-2).  The rule
# for them is therefore that of gpu_common.assert_close_storage: the device may be at most 1.5 times as far from
# the plain oracle as exact arithmetic with bf16 storage is (observed here: 0.9 .. 1.16 times).
QK_PATH = ("dX", "dk_accum", "dA[q]", "dB[q]", "dA[k]", "dB[k]")


def test_layer_c4_shape_all_targets():
    """One layer at the 14B shape (hidden 5120, 40 query / 8 kv heads, FFN 13824, qkv bias, LoRA on all
    seven projections) on a reduced token count the oracle finishes in seconds."""
    say("layer at the c4 (14B) shape")
    cfg = CONFIGS["c4_qwen14b_full"]
    batch = gen.batch_scaled(7, 6, 20, 300, [(0, 40, 40)], [(0, 48, 96)])
    run_layer_case(cfg, batch, ft_window=48, prefill_chunk=40, bwd_windows=[60, 36], seed=2, storage_exceptions=QK_PATH)


def test_layer_c5_shape_rank32():
    """One layer at the 32B shape (FFN 27648, LoRA rank 32 on all seven projections)."""
    say("layer at the c5 (32B) shape")
    cfg = CONFIGS["c5_qwen32b_full"]
    batch = gen.batch_scaled(8, 4, 20, 200, [(0, 24, 24)], [(0, 32, 64)])
    run_layer_case(cfg, batch, ft_window=32, prefill_chunk=24, bwd_windows=[40, 24], seed=3, storage_exceptions=QK_PATH)


# ------------------------------------------------------------------------------------------
# degenerate batches
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_name", ["c1", "small_bf16"])
def test_layer_inference_only_batches(cfg_name):
    """No finetune request in the batch (ft state = NULL): decode + prefill, then a single decode token."""
    cfg = C1 if cfg_name == "c1" else SMALL_BF16
    say(f"layer {cfg_name}: inference-only batches")
    tol = TOL[cfg.dtype]
    b = gen.mixed_batch(16, 31, decode_ctx=(1, 16, 17, 130), prefill=[(0, 33, 70), (48, 20, 90)], extra_capacity=2)
    b = gen.with_adapters(b, [0, -1])                                 # some inference requests use the adapter
    case = Case(cfg, b, seed=31)
    x = gen.layer_input(cfg, 31, b.n_tokens)
    y_g, y_o, _ = case.forward(b, x)
    assert_close("y", y_g, y_o, tol)
    one = gen.mixed_batch(16, 32, decode_ctx=(37,))                   # T = 1
    case = Case(cfg, one, seed=32)
    x = gen.layer_input(cfg, 32, 1)
    y_g, y_o, _ = case.forward(one, x)
    assert_close("y of a single token", y_g, y_o, tol)
    base = gen.mixed_batch(16, 33, decode_ctx=(5, 40), prefill=[(0, 18, 18)])   # nobody uses an adapter
    case = Case(cfg, base, seed=33)
    x = gen.layer_input(cfg, 33, base.n_tokens)
    y_g, y_o, _ = case.forward(base, x)
    assert_close("y without adapters", y_g, y_o, tol)


@pytest.mark.parametrize("cfg_name", ["c1", "small_bf16"])
def test_layer_finetune_only_windows_of_one_and_many(cfg_name):
    """The finetune sequence alone in the batch; forward windows 1 + 32 + rest, backward windows rest + 1 + 32."""
    cfg = C1 if cfg_name == "c1" else SMALL_BF16
    say(f"layer {cfg_name}: finetune-only batch, one-row windows")
    L = 49
    b = gen.mixed_batch(16, 34, finetune=[(0, 1, L)])
    tol = TOL[cfg.dtype]
    case = Case(cfg, b, seed=34)
    ft_seq = b.requests[0].seq_id
    x_seq = gen.layer_input(cfg, 34, L, tag="ftonly")
    y_g, y_o = np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden))
    start = 0
    for n_new in (1, 32, L - 33):
        bb = gen.Batch([gen.Request(KIND_FINETUNE, ft_seq, start, n_new, 0)], b.seq_pages, b.seq_capacity, b.num_pages,
                       b.page_size)
        g, o, _ = case.forward(bb, x_seq[start:start + n_new])
        y_g[start:start + n_new], y_o[start:start + n_new] = g, o
        start += n_new
    assert_close("y", y_g, y_o, tol)
    dY = gen.storage_round(cfg, gen.layer_input(cfg, 35, L, tag="dy"))
    grads_o = {}
    case.dev.zero_grads()
    case.d_ft[ft_seq].zero_accum()
    l = L
    dX_g, dX_o = np.zeros((L, cfg.hidden)), np.zeros((L, cfg.hidden))
    for s_ in (L - 33, 1, 32):
        g, o = case.backward_window(ft_seq, l - s_, s_, dY[l - s_:l], grads_o)
        dX_g[l - s_:l], dX_o[l - s_:l] = g, o
        l -= s_
    assert l == 0
    assert_close("dX", dX_g, dX_o, tol)
    grads_g = case.dev.grads_numpy()
    for t in cfg.lora_targets:
        assert_close(f"dA[{t}]", grads_g[t][0], grads_o[t][0], tol)
        assert_close(f"dB[{t}]", grads_g[t][1], grads_o[t][1], tol)


def test_layer_without_lora_targets():
    """cfg.lora_targets empty: the base model alone, forward and input gradient (lora = NULL)."""
    cfg = SMALL_BF16.with_(lora_targets=())
    say("layer small bf16 without LoRA targets")
    b = gen.batch_scaled(36, 4, 3, 200, [(0, 40, 40)], [(0, 70, 70)])
    case = Case(cfg, b, seed=36)
    x = gen.layer_input(cfg, 36, b.n_tokens)
    y_g, y_o, _ = case.forward(b, x)
    assert_close("y", y_g, y_o, TOL["bf16"])
    ft_seq = [r.seq_id for r in b.requests if r.kind == KIND_FINETUNE][0]
    dY = gen.storage_round(cfg, gen.layer_input(cfg, 37, 70, tag="dy"))
    case.d_ft[ft_seq].zero_accum()
    g, o = case.backward_window(ft_seq, 0, 70, dY, {})
    assert_close("dX", g, o, TOL["bf16"])


def test_forward_is_deterministic():
    say("determinism")
    case = Case(C1, gen.batch_c1(0))
    x = gen.layer_input(C1, 0, 68)
    y1, _, _ = case.forward(gen.batch_c1(0), x, oracle=False)
    y2, _, _ = case.forward(gen.batch_c1(0), x, oracle=False)
    assert np.array_equal(y1, y2)


def test_error_paths_on_device():
    say("error paths")
    case = Case(C1, gen.batch_c1(0))
    b = gen.batch_c1(0)
    db = HH.DeviceBatch(C1, b.requests, b.seq_pages, b.num_pages)
    x = torch.zeros((68, 256), device="cuda")
    y = torch.zeros_like(x)
    ws = HH.Workspace(case.dev.c, 68, db.host_maps.n_parts)
    ft = list(case.d_ft.values())[0]
    with pytest.raises(B.FlexcoError) as e:        # workspace too small
        B.flexco_layer_forward(case.dev.c, case.dev.w, case.dev.lora, db.maps, x, y, case.d_pool.c, ft.c, ws.ptr, 1024)
    assert e.value.code == B.FLEXCO_EWORKSPACE
    with pytest.raises(B.FlexcoError) as e:        # finetune request without its state
        B.flexco_layer_forward(case.dev.c, case.dev.w, case.dev.lora, db.maps, x, y, case.d_pool.c, None, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EINVAL
    with pytest.raises(B.FlexcoError) as e:        # aliasing
        B.flexco_layer_forward(case.dev.c, case.dev.w, case.dev.lora, db.maps, x, x, case.d_pool.c, ft.c, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EINVAL
    # maps whose page ids were checked against a larger pool than the one handed to the call
    big = HH.DeviceBatch(C1, b.requests, b.seq_pages, b.num_pages + 5)
    assert big.host_maps.num_pages == b.num_pages + 5 and db.host_maps.num_pages == b.num_pages
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_layer_forward(case.dev.c, case.dev.w, case.dev.lora, big.maps, x, y, case.d_pool.c, ft.c, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EPAGE
    q = torch.zeros((68, C1.q_dim), device="cuda")
    with pytest.raises(B.FlexcoError) as e:
        B.flexco_attention_mixed(case.dev.c, big.maps, q, case.d_pool.c, torch.empty_like(q), None, ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_EPAGE
    pages_d = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(B.FlexcoError) as e:        # window beyond the sequence
        B.flexco_lora_bwd(case.dev.c, case.dev.w, case.dev.lora, case.d_pool.c, pages_d, 4, ft.c, 60, 10, x, y,
                          ws.ptr, ws.bytes)
    assert e.value.code == B.FLEXCO_ESHAPE


def test_layer_c2_full_size_sampled():
    """The 8B-shaped configuration at full size, in the launch configuration bench.py times:
    the GPU runs the whole 1024-token batch; the oracle recomputes a sample of requests
    (16 decode, both prefill chunks, the finetune window) one by one from the same inputs."""
    say("layer c2 full size, sampled")
    full_size_sampled(C2, gen.batch_c2(0), 16)


@pytest.mark.parametrize("name,make_batch,n_decode", [
    ("c3_llama8b_full", gen.batch_c3, 16),
    ("c4_qwen14b_full", gen.batch_c4, 8),
    ("c5_qwen32b_full", gen.batch_c5, 8),
])
def test_layer_whole_model_batches_full_size_sampled(name, make_batch, n_decode):
    """One layer of the 8B / 14B / 32B-shaped models on the whole-model configurations' full batches
    (T = 2048 / 2048 / 4096, windows of 512 / 1024 / 1024 rows on prefixes of 1536 / 3072 / 3072), sampled
    like the benchmark configuration's case."""
    say("layer %s full size, sampled" % name)
    full_size_sampled(CONFIGS[name], make_batch(0), n_decode)


@pytest.mark.parametrize("share", [0.25, 0.75, 0.9])
def test_layer_c4_inference_share_sweep_full_size_sampled(share):
    """The 14B-shaped layer on the token budget of 2048 at the other inference shares of the configuration
    (finetune windows of 1536 / 512 / 205 rows at the end of a 4096-token sequence; 50 % is the case above)."""
    say("layer c4 full size at inference share %.2f, sampled" % share)
    full_size_sampled(CONFIGS["c4_qwen14b_full"], gen.batch_c4(0, share), 6)


def test_layer_c4_decode_free_iteration_full_size():
    """An iteration without inference decode tokens at the 14B shape (a whole 512-token prompt and the 1024-row
    finetune window on its 3072-row prefix): the attention's chunk items then run on the four-wavefront kernel alone, in
    its three-stage form; every request goes through the oracle."""
    say("layer c4, decode-free iteration, full size")
    cfg = CONFIGS["c4_qwen14b_full"]
    batch = gen.mixed_batch(cfg.page_size, 0, decode_ctx=(), prefill=[(0, 512, 512)], finetune=[(3072, 1024, 4096)])
    full_size_sampled(cfg, batch, 0)


def full_size_sampled(cfg, batch, n_decode):
    seed = 0
    tol = TOL["bf16"]
    W, lora = gen.layer_weights(cfg, seed, 0), gen.lora_weights(cfg, seed, 0)
    dev = HH.DeviceLayer(cfg, W, lora)
    pool = HH.DevicePool(cfg, batch.num_pages)
    pool.fill_random(seed)
    sample = gen.sample_requests(batch, n_decode)
    o_pool = OL.KVPool(batch.num_pages, cfg.page_size, cfg.kv_dim, dtype=np.float32)
    for r in sample:
        if r.start_pos:
            k, v = gen.kv_prefix(cfg, seed, 0, r.seq_id, r.start_pos)
            pool.write_rows(batch.seq_pages[r.seq_id], k, v)
            sl = o_pool.slots(batch.seq_pages[r.seq_id], r.start_pos)
            o_pool.k[sl], o_pool.v[sl] = k, v
    ft_req = [r for r in batch.requests if r.kind == KIND_FINETUNE][0]
    L = batch.seq_capacity[ft_req.seq_id]
    ft = HH.DeviceFtState(cfg, L)
    db = HH.DeviceBatch(cfg, batch.requests, batch.seq_pages, batch.num_pages)
    ws = HH.Workspace(dev.c, db.host_maps.T, db.host_maps.n_parts, ft_req.n_new, L)
    x_np = gen.layer_input(cfg, seed, db.host_maps.T)
    x = torch.from_numpy(x_np).to("cuda", torch.bfloat16)
    y = torch.empty_like(x)
    say("  gpu forward")
    B.flexco_layer_forward(dev.c, dev.w, dev.lora, db.maps, x, y, pool.c, ft.c, ws.ptr, ws.bytes)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y).all()), "a row of the full batch's output is not finite"      # all T rows, sampled or not
    rows = gen.sample_token_rows(batch, sample)
    om = build_maps(sample, batch.seq_pages, batch.page_size, batch.num_pages)
    o_ft = {ft_req.seq_id: OL.FtState(cfg, L)}
    say("  oracle forward on %d sampled tokens (%d requests, prefill chunks at %s)" % (
        len(rows), len(sample), [r.start_pos for r in sample if r.kind == 1]))
    y_o = OL.layer_forward_mixed(cfg, W, lora, om, x_np[rows], o_pool, o_ft)
    report, elem = [], []

    def check(name, got, ref):
        assert_close(name, got, ref, tol, report)
        elem.append((name, elem_err(got, ref, tol)))

    y_g = to_np(y)[rows]
    check("y (sampled rows)", y_g, y_o)
    off = 0
    for r in sample:                                   # every kind of request on its own as well
        if r.kind != 0:
            check("y of request kind %d at %d" % (r.kind, r.start_pos), y_g[off:off + r.n_new], y_o[off:off + r.n_new])
        off += r.n_new
    w = slice(ft_req.start_pos, ft_req.start_pos + ft_req.n_new)
    for name in ("q_cache", "x", "x2", "gate", "up", "attn", "lse"):
        check("saved " + name, to_np(getattr(ft, name))[w], getattr(o_ft[ft_req.seq_id], name)[w])
    say("  backward window")
    dY_np = gen.layer_input(cfg, seed, ft_req.n_new, tag="dy")
    dY = torch.from_numpy(dY_np).to("cuda", torch.bfloat16)
    dX = torch.empty_like(dY)
    pages_d = torch.from_numpy(np.asarray(batch.seq_pages[ft_req.seq_id], dtype=np.int32)).to("cuda")
    B.flexco_lora_bwd(dev.c, dev.w, dev.lora, pool.c, pages_d, int(pages_d.numel()), ft.c, ft_req.start_pos,
                      ft_req.n_new, dY, dX, ws.ptr, ws.bytes)
    torch.cuda.synchronize()
    sl = o_pool.slots(batch.seq_pages[ft_req.seq_id], L)
    grads_o = {}
    dX_o = OL.layer_backward_window(cfg, W, lora, o_ft[ft_req.seq_id], o_pool.k[sl].astype(np.float64),
                                    o_pool.v[sl].astype(np.float64), ft_req.start_pos, ft_req.n_new, dY_np, grads_o)
    check("dX", to_np(dX), dX_o)
    check("dk_accum", to_np(ft.dk_accum), o_ft[ft_req.seq_id].dk_accum)
    check("dv_accum", to_np(ft.dv_accum), o_ft[ft_req.seq_id].dv_accum)
    grads_g = dev.grads_numpy()
    for t in cfg.lora_targets:
        check(f"dA[{t}]", grads_g[t][0], grads_o[t][0])
        check(f"dB[{t}]", grads_g[t][1], grads_o[t][1])
    say("  max-norm: " + ", ".join(f"{n}={e:.1e}" for n, e in report))
    # elementwise: |gpu - oracle| <= 1e-3 max|oracle| + 2e-2 |oracle| for every element would be a worst ratio <= 1.
    # Reported, and bounded loosely: an element near zero of a tensor whose rows are sums of many bf16 products
    # carries the absolute error of its row, so single elements sit above 1 while the tensor as a whole is
    # within 2e-2 of its largest value.
    say("  elementwise worst |d| / (1e-3 max + 2e-2 |ref|): " + ", ".join(f"{n}={e:.2f}" for n, e in elem))
    assert max(e for _, e in elem) <= 20.0, elem
