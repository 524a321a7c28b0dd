"""Pins for oracle/layer.py: the four properties (LoRA with B = 0 is the base layer;
token-level == whole-sequence; gradients == central finite differences; attention
== brute force, see test_oracle_ops.py) plus a whole-layer cross-check against a
library-routine implementation with reverse-mode autodiff."""
from types import SimpleNamespace as NS

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layer as L
from oracle.maps import build_maps
from workload import gen, target_dims, CONFIGS
from helpers import SMALL, small_layer, rel_err

RNG = np.random.default_rng(11)


def seq_input(cfg, n, seed=3):
    return gen.rng(seed, "xin", n).standard_normal((n, cfg.hidden))


# ---- property 1: B = 0 ----------------------------------------------------------
def test_lora_with_zero_B_is_base_layer():
    cfg = SMALL
    W, lo = small_layer()
    lo0 = {t: (A, np.zeros_like(B)) for t, (A, B) in lo.items()}
    x = seq_input(cfg, 12)
    base = L.layer_forward_seq(cfg, W, None, x)
    with0 = L.layer_forward_seq(cfg, W, lo0, x)
    assert np.array_equal(base["y"], with0["y"])
    dY = RNG.standard_normal(x.shape)
    _, grads, _, _ = L.layer_backward_seq(cfg, W, lo0, x, dY)
    for t, (dA, dB) in grads.items():
        assert np.all(dA == 0.0), t
        assert np.any(dB != 0.0), t
    # and a non-zero B does change the output
    assert not np.array_equal(base["y"], L.layer_forward_seq(cfg, W, lo, x)["y"])


def test_zero_weights_give_identity_residual():
    cfg = SMALL
    W, _ = small_layer()
    Wz = {k: (np.zeros_like(v) if k.startswith("w") or k.startswith("b") else v) for k, v in W.items()}
    x = seq_input(cfg, 5)
    assert np.array_equal(L.layer_forward_seq(cfg, Wz, None, x)["y"], x)


# ---- whole layer vs library routines + autograd ---------------------------------
def torch_layer(cfg, W, lo, x):
    """Independent whole-sequence layer from torch library ops (F.linear, F.rms_norm,
    F.scaled_dot_product_attention, F.silu); complex-number rotary embedding."""
    n = x.shape[0]
    s = cfg.lora_scale

    def lin(t, w, b, name):
        y = F.linear(t, W[w], W.get(b) if b else None)
        if name in lo:
            y = y + s * (t @ lo[name][0]) @ lo[name][1]
        return y

    def rot(t, nh):
        d = cfg.head_dim
        th = t.reshape(n, nh, d)
        zc = torch.complex(th[..., :d // 2], th[..., d // 2:])
        freqs = cfg.rope_theta ** (-torch.arange(0, d // 2, dtype=torch.float64) * 2 / d)
        ang = torch.arange(n, dtype=torch.float64)[:, None] * freqs[None, :]
        zr = zc * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([zr.real, zr.imag], dim=-1)

    h1 = F.rms_norm(x, (cfg.hidden,), W["g1"], eps=cfg.rms_eps)
    q = rot(lin(h1, "wq", "bq", "q"), cfg.n_q_heads).transpose(0, 1)[None]
    k = rot(lin(h1, "wk", "bk", "k"), cfg.n_kv_heads).transpose(0, 1)[None]
    v = lin(h1, "wv", "bv", "v").reshape(n, cfg.n_kv_heads, cfg.head_dim).transpose(0, 1)[None]
    a = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)
    a = a[0].transpose(0, 1).reshape(n, cfg.q_dim)
    x2 = x + lin(a, "wo", None, "o")
    h2 = F.rms_norm(x2, (cfg.hidden,), W["g2"], eps=cfg.rms_eps)
    act = F.silu(lin(h2, "wg", None, "gate")) * lin(h2, "wu", None, "up")
    return x2 + lin(act, "wd", None, "down")


@pytest.mark.parametrize("targets", [("q", "k", "v", "o", "gate", "up", "down"), ("q", "v", "down"), ("down",)])
def test_layer_matches_library_autograd(targets):
    cfg = SMALL.with_(lora_targets=targets)
    W, lo = small_layer(cfg)
    n = 10
    x = seq_input(cfg, n)
    tgt = RNG.standard_normal(x.shape)
    tW = {k: torch.from_numpy(v) for k, v in W.items()}
    tlo = {t: (torch.from_numpy(A).requires_grad_(), torch.from_numpy(B).requires_grad_()) for t, (A, B) in lo.items()}
    tx = torch.from_numpy(x).requires_grad_()
    ty = torch_layer(cfg, tW, tlo, tx)
    loss = torch.mean((ty - torch.from_numpy(tgt)) ** 2)
    loss.backward()
    o_loss, o_grads, o_dx = L.finetune_whole_seq(cfg, [W], [lo], x, tgt)
    assert abs(o_loss - loss.item()) < 1e-12 * max(1.0, abs(loss.item()))
    assert rel_err(o_dx, tx.grad.numpy()) < 1e-10
    assert set(o_grads[0]) == set(targets)
    for t in targets:
        assert rel_err(o_grads[0][t][0], tlo[t][0].grad.numpy()) < 1e-10, t
        assert rel_err(o_grads[0][t][1], tlo[t][1].grad.numpy()) < 1e-10, t


# ---- property 3: finite differences ----------------------------------------------
def test_gradients_match_central_finite_differences():
    cfg = SMALL
    W, lo = small_layer()
    n = 7
    x = seq_input(cfg, n)
    tgt = RNG.standard_normal(x.shape)
    _, grads, dx = L.finetune_whole_seq(cfg, [W], [lo], x, tgt)
    loss = lambda: L.mse_loss_grad(L.layer_forward_seq(cfg, W, lo, x)["y"], tgt)[0]
    h = 1e-6

    def check(arr, ana, k=4):
        flat = arr.reshape(-1)
        for i in RNG.choice(flat.size, size=k, replace=False):
            old = flat[i]
            flat[i] = old + h
            fp = loss()
            flat[i] = old - h
            fm = loss()
            flat[i] = old
            num = (fp - fm) / (2 * h)
            assert abs(num - ana.reshape(-1)[i]) <= 1e-6 * max(abs(num), abs(ana.reshape(-1)[i])) + 1e-9

    check(x, dx, 6)
    for t, (A, B) in lo.items():
        check(A, grads[0][t][0])
        check(B, grads[0][t][1])


# ---- property 2: token-level == whole sequence -------------------------------------
SPLITS = [
    ([12], [12]),
    ([1] * 12, [1] * 12),
    ([4, 4, 4], [4, 4, 4]),
    ([5, 7], [3, 2, 7]),            # forward and backward splits differ
    ([7, 1, 4], [12]),
    ([12], [2, 9, 1]),
]


@pytest.mark.parametrize("fwd,bwd", SPLITS)
def test_token_level_equals_whole_sequence(fwd, bwd):
    cfg = SMALL
    W, lo = small_layer()
    W2, lo2 = small_layer(seed=2, layer=1)
    n = 12
    x = seq_input(cfg, n)
    tgt = RNG.standard_normal(x.shape)
    loss_w, grads_w, dx_w = L.finetune_whole_seq(cfg, [W, W2], [lo, lo2], x, tgt)
    pages = np.array([5, 0, 3])     # scattered pages, page size 4
    loss_t, grads_t, dx_t, states = L.finetune_token_level(cfg, [W, W2], [lo, lo2], x, tgt, fwd, bwd,
                                                          page_size=4, pages=pages)
    assert abs(loss_w - loss_t) < 1e-13
    assert rel_err(dx_t, dx_w) < 1e-11
    for n_ in range(2):
        for t in cfg.lora_targets:
            assert rel_err(grads_t[n_][t][0], grads_w[n_][t][0]) < 1e-11
            assert rel_err(grads_t[n_][t][1], grads_w[n_][t][1]) < 1e-11


def test_kv_gradient_accumulator_equals_whole_sequence_dk_dv():
    cfg = SMALL
    W, lo = small_layer()
    n = 9
    x = seq_input(cfg, n)
    tgt = RNG.standard_normal(x.shape)
    _, dY = L.mse_loss_grad(L.layer_forward_seq(cfg, W, lo, x)["y"], tgt)
    _, _, dK, dV = L.layer_backward_seq(cfg, W, lo, x, dY)
    _, _, _, states = L.finetune_token_level(cfg, [W], [lo], x, tgt, [4, 5], [2, 3, 4], page_size=4)
    assert rel_err(states[0].dk_accum, dK) < 1e-11
    assert rel_err(states[0].dv_accum, dV) < 1e-11
    assert states[0].q_cache.shape == (n, cfg.q_dim)          # dQ rows per window, dK/dV rows up to its end


def test_backward_without_input_grad():
    cfg = SMALL.with_(lora_targets=("down",))
    W, lo = small_layer(cfg)
    x = seq_input(cfg, 6)
    tgt = RNG.standard_normal(x.shape)
    _, g_w, _ = L.finetune_whole_seq(cfg, [W], [lo], x, tgt)
    _, _, _, states = L.finetune_token_level(cfg, [W], [lo], x, tgt, [6], [6], page_size=4)
    _, dY = L.mse_loss_grad(L.layer_forward_seq(cfg, W, lo, x)["y"], tgt)
    grads = {}
    st = states[0]
    st.dk_accum[:] = 0
    st.dv_accum[:] = 0
    f = L.layer_forward_seq(cfg, W, lo, x)
    out = L.layer_backward_window(cfg, W, lo, st, f["k"], f["v"], 0, 6, dY, grads, need_dx=False)
    assert out is None
    assert rel_err(grads["down"][0], g_w[0]["down"][0]) < 1e-12


# ---- mixed batch through the caches ---------------------------------------------------
def _run_chunks(cfg, W, lo, x, chunks, pages, kind=1, adapter=-1, page_size=4):
    pool = L.KVPool(int(max(pages)) + 1, page_size, cfg.kv_dim)
    out, l = [], 0
    for s in chunks:
        maps = build_maps([NS(kind=kind, seq_id=0, start_pos=l, n_new=s, adapter=adapter)], {0: pages}, page_size)
        out.append(L.layer_forward_mixed(cfg, W, lo, maps, x[l:l + s], pool))
        l += s
    return np.concatenate(out), pool


def test_chunked_prefill_equals_unchunked_equals_decode():
    cfg = SMALL
    W, lo = small_layer()
    n = 11
    x = seq_input(cfg, n)
    whole = L.layer_forward_seq(cfg, W, None, x)["y"]
    for chunks in ([11], [4, 7], [1] * 11, [8, 1, 1, 1]):
        y, _ = _run_chunks(cfg, W, lo, x, chunks, [2, 0, 1])
        assert rel_err(y, whole) < 1e-12, chunks
    # finetune rows follow the same pattern as prefill rows, with the adapter on
    whole_l = L.layer_forward_seq(cfg, W, lo, x)["y"]
    y, _ = _run_chunks(cfg, W, lo, x, [3, 8], [2, 0, 1], kind=2, adapter=0)
    assert rel_err(y, whole_l) < 1e-12


def test_page_permutation_is_bit_invariant():
    cfg = SMALL
    W, lo = small_layer()
    x = seq_input(cfg, 10)
    y1, _ = _run_chunks(cfg, W, lo, x, [6, 4], [0, 1, 2])
    y2, _ = _run_chunks(cfg, W, lo, x, [6, 4], [7, 2, 4])
    assert np.array_equal(y1, y2)


def test_mixed_batch_rows_equal_per_sequence_definition():
    """decode + prefill + finetune rows in ONE batch equal the whole-sequence
    definition of each sequence; inference rows do not see the adapter."""
    cfg = SMALL
    W, lo = small_layer()
    ps = 4
    xs = {0: seq_input(cfg, 9, seed=20), 1: seq_input(cfg, 6, seed=21), 2: seq_input(cfg, 8, seed=22)}
    pages = {0: [4, 1, 6], 1: [0, 5], 2: [3, 2]}
    pool = L.KVPool(8, ps, cfg.kv_dim)
    # iteration 0 fills the prefixes: seq 0 rows 0..7 (prefill), seq 2 rows 0..3 (finetune window 0)
    m0 = build_maps([NS(kind=1, seq_id=0, start_pos=0, n_new=8, adapter=-1),
                     NS(kind=2, seq_id=2, start_pos=0, n_new=4, adapter=0)], pages, ps)
    st = {2: L.FtState(cfg, 8)}
    L.layer_forward_mixed(cfg, W, lo, m0, np.concatenate([xs[0][:8], xs[2][:4]]), pool, st)
    # iteration 1: decode token of seq 0, prefill chunk of seq 1, finetune window 1 of seq 2
    m1 = build_maps([NS(kind=0, seq_id=0, start_pos=8, n_new=1, adapter=-1),
                     NS(kind=1, seq_id=1, start_pos=0, n_new=6, adapter=-1),
                     NS(kind=2, seq_id=2, start_pos=4, n_new=4, adapter=0)], pages, ps)
    y = L.layer_forward_mixed(cfg, W, lo, m1, np.concatenate([xs[0][8:], xs[1], xs[2][4:]]), pool, st)
    assert rel_err(y[0:1], L.layer_forward_seq(cfg, W, None, xs[0])["y"][8:]) < 1e-12
    assert rel_err(y[1:7], L.layer_forward_seq(cfg, W, None, xs[1])["y"]) < 1e-12
    ft = L.layer_forward_seq(cfg, W, lo, xs[2])
    assert rel_err(y[7:], ft["y"][4:]) < 1e-12
    for name, ref in (("q_cache", "q"), ("x2", "x2"), ("gate", "gate"), ("up", "up"), ("attn", "a"), ("lse", "lse")):
        assert rel_err(getattr(st[2], name), ft[ref]) < 1e-12, name
    # inference rows are untouched by the adapter's values
    lo_b = {t: (A * 3.0, B * -2.0) for t, (A, B) in lo.items()}
    pool2 = L.KVPool(8, ps, cfg.kv_dim)
    pool2.k[:], pool2.v[:] = pool.k, pool.v
    y_b = L.layer_forward_mixed(cfg, W, lo_b, m1, np.concatenate([xs[0][8:], xs[1], xs[2][4:]]), pool2, None)
    assert np.array_equal(y_b[:7], y[:7]) and not np.array_equal(y_b[7:], y[7:])


def test_several_adapters_in_one_batch_equal_each_sequence_with_its_own_adapter():
    """Requests served by different adapters (and by none) in ONE batch: every request's rows equal the
    whole-sequence definition of its sequence under its own adapter (Sec. 6.2, co-served PEFT models)."""
    cfg = SMALL
    W, lo0 = small_layer()
    lo1 = {t: (A[::-1].copy() * 1.5, B[:, ::-1].copy() * -2.0) for t, (A, B) in lo0.items()}
    lo2 = {t: (A * -0.7, B * 3.0) for t, (A, B) in lo0.items()}
    adapters = [lo0, lo1, lo2]
    ps = 4
    lens = {0: 9, 1: 6, 2: 8, 3: 5}
    xs = {s: seq_input(cfg, n, seed=30 + s) for s, n in lens.items()}
    pages = {0: [4, 1, 6], 1: [0, 5], 2: [3, 2], 3: [7, 8]}
    pool = L.KVPool(9, ps, cfg.kv_dim)
    # iteration 0: prefixes under each sequence's adapter (seq 0: adapter 1, seq 3: adapter 2)
    m0 = build_maps([NS(kind=1, seq_id=0, start_pos=0, n_new=8, adapter=1),
                     NS(kind=1, seq_id=3, start_pos=0, n_new=4, adapter=2),
                     NS(kind=2, seq_id=2, start_pos=0, n_new=4, adapter=0)], pages, ps)
    st = {2: L.FtState(cfg, 8)}
    L.layer_forward_mixed(cfg, W, adapters, m0, np.concatenate([xs[0][:8], xs[3][:4], xs[2][:4]]), pool, st)
    # iteration 1: decode of seq 0 (adapter 1), prefill of seq 1 (no adapter), decode of seq 3 (adapter 2),
    # finetune window of seq 2 (adapter 0)
    m1 = build_maps([NS(kind=0, seq_id=0, start_pos=8, n_new=1, adapter=1),
                     NS(kind=1, seq_id=1, start_pos=0, n_new=6, adapter=-1),
                     NS(kind=0, seq_id=3, start_pos=4, n_new=1, adapter=2),
                     NS(kind=2, seq_id=2, start_pos=4, n_new=4, adapter=0)], pages, ps)
    y = L.layer_forward_mixed(cfg, W, adapters, m1, np.concatenate([xs[0][8:], xs[1], xs[3][4:], xs[2][4:]]), pool, st)
    assert rel_err(y[0:1], L.layer_forward_seq(cfg, W, lo1, xs[0])["y"][8:]) < 1e-12
    assert rel_err(y[1:7], L.layer_forward_seq(cfg, W, None, xs[1])["y"]) < 1e-12
    assert rel_err(y[7:8], L.layer_forward_seq(cfg, W, lo2, xs[3])["y"][4:]) < 1e-12
    assert rel_err(y[8:], L.layer_forward_seq(cfg, W, lo0, xs[2])["y"][4:]) < 1e-12
    # a wrong assignment is visible: seq 0 under adapter 2 differs
    assert rel_err(y[0:1], L.layer_forward_seq(cfg, W, lo2, xs[0])["y"][8:]) > 1e-6


def test_rope_makes_attention_shift_invariant():
    """Shifting every position of a sequence by a constant leaves the attention
    output unchanged (rotary embedding is relative)."""
    from oracle import ops
    cfg = SMALL
    n, nq, nkv, d = 6, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    q0, k0 = RNG.standard_normal((n, nq * d)), RNG.standard_normal((n, nkv * d))
    v = RNG.standard_normal((n, nkv * d))
    outs = []
    for shift in (0, 37):
        pos = np.arange(n) + shift
        q, k = ops.rope(q0, pos, nq, d, cfg.rope_theta), ops.rope(k0, pos, nkv, d, cfg.rope_theta)
        outs.append(ops.attention(q, np.arange(n), k, v, nq, nkv, d)[0])
    assert np.allclose(outs[0], outs[1], atol=1e-11)


# ---- closed forms ------------------------------------------------------------------------
def test_mse_closed_form():
    y, t = np.array([[1.0, 2.0], [3.0, 5.0]]), np.array([[0.0, 2.0], [1.0, 1.0]])
    loss, d = L.mse_loss_grad(y, t)
    assert loss == (1.0 + 0.0 + 4.0 + 16.0) / 4.0
    assert np.array_equal(d, 2.0 * (y - t) / 4.0)


def test_lora_parameter_counts_match_paper():
    """Sec. 8 (LLMs and PEFT models): rank-16 LoRA on the down projections has 9.4M
    (LLaMA-3.1-8B) and 14.5M (Qwen-2.5-14B) trainable parameters; with A [in, r] and
    B [r, out] that is r * (ffn + hidden) * layers."""
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "lora_trainable_parameters.txt"))
            if l.strip() and not l.startswith("#")]
    printed = [(r[0], float(r[1])) for r in rows if len(r) == 2]
    assert len(printed) == 2
    for name, millions in printed:
        cfg = CONFIGS[name].with_(lora_targets=("down",), lora_rank=16)
        lo = {t: target_dims(cfg, t) for t in cfg.lora_targets}
        count = sum(cfg.lora_rank * (i + o) for i, o in lo.values()) * cfg.n_layers
        assert round(count / 1e6, 1) == millions
    cfg = CONFIGS["c1_tiny_f32"]
    lw = gen.lora_weights(cfg, 0)
    assert lw["down"][0].shape == (cfg.ffn, cfg.lora_rank) and lw["down"][1].shape == (cfg.lora_rank, cfg.hidden)


# ---- storage rounding mode -------------------------------------------------------------
def test_round_bf16_is_the_format_rounding():
    """hand values (spacing at 1.0 is 2^-7; ties go to the even significand) and the library's conversion"""
    from oracle import ops
    one = 1.0
    hand = [(one, one), (one + 2.0 ** -8, one), (one + 3 * 2.0 ** -8, one + 2.0 ** -6), (one + 2.0 ** -7, one + 2.0 ** -7),
            (one + 2.0 ** -8 + 2.0 ** -20, one + 2.0 ** -7), (-3.0 - 2.0 ** -7, -3.0), (-3.0 - 2.0 ** -6, -3.0 - 2.0 ** -6), (0.0, 0.0),
            (2.0 - 2.0 ** -9, 2.0), (255.5, 256.0), (1e-3, 131.0 / 128.0 * 2.0 ** -10)]
    for a, want in hand:
        assert ops.round_bf16(np.array([a]))[0] == want, a
    a = np.concatenate([RNG.standard_normal(20000) * s for s in (1e-6, 1e-2, 1.0, 77.0, 3e5)])
    lib = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).double().numpy()
    assert np.array_equal(ops.round_bf16(a.astype(np.float32)).astype(np.float64), lib)
    assert ops.round_bf16(a).dtype == np.float64          # the input's own type comes back
    assert np.array_equal(ops.round_bf16(ops.round_bf16(a)), ops.round_bf16(a))     # idempotent


def _token_level_once(cfg, W, lo, x, dY, fwd, bwd, storage):
    """Alg. 2 for one sequence alone: forward windows, then backward windows from the end, with `storage`."""
    n = x.shape[0]
    pages = np.array([5, 0, 3, 1])
    pool = L.KVPool(int(pages.max()) + 1, 4, cfg.kv_dim)
    st = L.FtState(cfg, n)
    y, l = np.zeros_like(x), 0
    for s in fwd:
        maps = build_maps([NS(kind=2, seq_id=0, start_pos=l, n_new=s, adapter=0)], {0: pages}, 4)
        y[l:l + s] = L.layer_forward_mixed(cfg, W, lo, maps, x[l:l + s], pool, {0: st}, storage=storage)
        l += s
    grads, dx, l = {}, np.zeros_like(x), n
    slots = pool.slots(pages, n)
    for s in bwd:
        dx[l - s:l] = L.layer_backward_window(cfg, W, lo, st, pool.k[slots[:l]], pool.v[slots[:l]], l - s, s,
                                              dY[l - s:l], grads, storage=storage)
        l -= s
    return y, dx, grads, st, pool


def test_storage_mode_none_and_identity_are_the_plain_method():
    cfg = SMALL
    W, lo = small_layer()
    x, dY = seq_input(cfg, 14), RNG.standard_normal((14, cfg.hidden))
    plain = _token_level_once(cfg, W, lo, x, dY, [5, 9], [4, 10], None)
    ident = _token_level_once(cfg, W, lo, x, dY, [5, 9], [4, 10], lambda a: a)
    f32 = _token_level_once(cfg, W, lo, x, dY, [5, 9], [4, 10], lambda a: np.asarray(a, dtype=np.float64))
    for other in (ident, f32):
        assert np.array_equal(plain[0], other[0]) and np.array_equal(plain[1], other[1])
        for t in cfg.lora_targets:
            assert np.array_equal(plain[2][t][0], other[2][t][0]) and np.array_equal(plain[2][t][1], other[2][t][1])
    # and the plain method is the definition (so the switch did not disturb it)
    dX_w, grads_w, _, _ = L.layer_backward_seq(cfg, W, lo, x, dY)
    assert rel_err(plain[1], dX_w) < 1e-11
    assert rel_err(plain[0], L.layer_forward_seq(cfg, W, lo, x)["y"]) < 1e-12


def test_storage_mode_rounds_what_is_stored_and_stays_near_the_plain_method():
    """Every tensor the state and the pool hold, and both results, are representable in the storage type;
    accumulators are not rounded; the distance to the unrounded method is a small multiple of the
    format's 2^-9 relative rounding (a layer output passes about ten roundings in sequence) - and not zero."""
    from oracle import ops
    cfg = SMALL
    W, lo = small_layer()
    rb = lambda a: ops.round_bf16(np.asarray(a, dtype=np.float64))
    W = {k: rb(v) for k, v in W.items()}
    lo = {t: (rb(A), rb(B)) for t, (A, B) in lo.items()}
    x, dY = rb(seq_input(cfg, 14)), rb(RNG.standard_normal((14, cfg.hidden)))
    y0, dx0, g0, st0, _ = _token_level_once(cfg, W, lo, x, dY, [5, 9], [4, 10], None)
    y1, dx1, g1, st1, pool1 = _token_level_once(cfg, W, lo, x, dY, [5, 9], [4, 10], "bf16")
    for name, t in (("y", y1), ("dx", dx1), ("q_cache", st1.q_cache), ("x2", st1.x2), ("gate", st1.gate), ("up", st1.up),
                    ("attn", st1.attn), ("k", pool1.k), ("v", pool1.v)):
        assert np.array_equal(rb(t), t), name
    assert not np.array_equal(rb(st1.lse), st1.lse) and not np.array_equal(rb(st1.dk_accum), st1.dk_accum)
    u = 2.0 ** -9
    for name, a, b, k in (("y", y1, y0, 8), ("dx", dx1, dx0, 16), ("q_cache", st1.q_cache, st0.q_cache, 4),
                          ("dk_accum", st1.dk_accum, st0.dk_accum, 16)):
        e = rel_err(a, b)
        assert 0.05 * u < e <= k * u, (name, e)
    for t in cfg.lora_targets:
        for i in (0, 1):
            e = rel_err(g1[t][i], g0[t][i])
            assert 0.0 < e <= 24 * u, (t, i, e)
    # a callable does the same as the name
    y2, dx2, _, _, _ = _token_level_once(cfg, W, lo, x, dY, [5, 9], [4, 10], rb)
    assert np.array_equal(y2, y1) and np.array_equal(dx2, dx1)
    # window splits no longer give bit-equal results (rounded intermediates), but stay as near
    y3, dx3, _, _, _ = _token_level_once(cfg, W, lo, x, dY, [14], [14], "bf16")
    assert rel_err(y3, y1) <= 8 * u and rel_err(dx3, dx1) <= 16 * u


def test_bf16_storage_alone_misses_2e2_on_the_logit_path_of_the_short_14b_case():
    """Evidence for the one exception of the GPU parity tests (the 14B / 32B shapes on <= 96 keys): the oracle with
    EXACT fp64 arithmetic and bf16 storage is itself more than 2e-2 away from the unrounded oracle on the tensors
    that depend on the gradient through the softmax logits, and well inside on all the others; and two such runs
    that differ only in arithmetic precision (fp64 / fp32: both correct implementations of the same storage type)
    already differ from each other by several 1e-3, which is why a device result cannot be held to the storage
    oracle itself much tighter than to the plain one."""
    from helpers import oracle_layer_case, oracle_layer_case_backward
    from workload import CONFIGS
    cfg = CONFIGS["c4_qwen14b_full"]
    b0 = gen.batch_scaled(7, 6, 20, 300, [(0, 40, 40)], [(0, 48, 96)])
    kw = dict(ft_window=48, prefill_chunk=40, bwd_windows=[60, 36])
    plain, st = oracle_layer_case(cfg, b0, seed=2, **kw)
    Ls = st[5]
    _, dY = L.mse_loss_grad(plain["y_ft"], gen.loss_targets(cfg, 2, Ls).astype(np.float64))
    dY = gen.storage_round(cfg, (dY * Ls * cfg.hidden).astype(np.float32)).astype(np.float64)
    plain.update(oracle_layer_case_backward(cfg, b0, kw["bwd_windows"], 2, st, dY))
    runs = {}
    for label, dt in (("s64", np.float64), ("s32", np.float32)):
        f, st = oracle_layer_case(cfg, b0, seed=2, storage="bf16", dtype=dt, **kw)
        f.update(oracle_layer_case_backward(cfg, b0, kw["bwd_windows"], 2, st, dY, storage="bf16", dtype=dt))
        runs[label] = f
    logit_path = ("dX", "dk_accum", "dA[q]", "dB[q]", "dA[k]", "dB[k]")
    for name in plain:
        if name == "y_ft" or name == "saved x":
            continue
        e64 = rel_err(runs["s64"][name], plain[name])
        e32_64 = rel_err(runs["s32"][name], runs["s64"][name])
        if name in logit_path:
            assert 2e-2 < e64 < 4e-2, (name, e64)
        else:
            assert e64 < 1e-2, (name, e64)
        assert e32_64 < 1e-2, (name, e32_64)
    assert max(rel_err(runs["s32"][n], runs["s64"][n]) for n in logit_path) > 2e-3
