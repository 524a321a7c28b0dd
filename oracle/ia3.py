"""A decoder layer with an (IA)^3 bypass network: definition and the token-level method
(oracle side; test infrastructure).

Sec. 4.1 gives (IA)^3 as the example of a PEFT method that changes the backbone's topology by an
elementwise product and still fits the bypass form: with a learned vector l, Y = X (.) l is written
Y = X + X (.) (l - 1), a bypass network X (.) (l - 1) added to the backbone tensor X.  (IA)^3 itself
(Liu et al., 2022) places three such vectors per layer: on the key projection's output, on the value
projection's output and on the inner activation of the feed-forward block, here the SwiGLU product
that the down projection reads.  Readings: the key is scaled before its rotation (the bypass sits on
the projection's output, like a LoRA bypass); only rows of requests that carry the adapter are
scaled; the vectors are the only trainable parameters.

Like oracle/layer.py there are two ways to the same numbers: the whole-sequence definition with a
hand-derived backward pass, and Algorithm 2's windows over the caches reading only what graph
pruning (Alg. 1) keeps - for this network x, x2, gate, up, Q, K, V plus the unscaled key and value
rows (the other operand of a product whose gradient is wanted); the SwiGLU product is recomputed.
"""
import numpy as np

from . import ops
from .layer import FtState, _cast, attention_mixed


def bypass_scale(t, l, rows):
    """Y = X + X (.) (l - 1) on the adapter's rows, Y = X elsewhere (Sec. 4.1)."""
    y = t.copy()
    y[rows] = t[rows] + t[rows] * (l - 1.0)
    return y


class Ia3FtState(FtState):
    """FtState plus the unscaled key/value rows of the finetune sequence."""

    def __init__(self, cfg, L, dtype=np.float64):
        super().__init__(cfg, L, dtype)
        self.k0 = np.zeros((L, cfg.kv_dim), dtype=dtype)
        self.v0 = np.zeros((L, cfg.kv_dim), dtype=dtype)


def _base(W, xin, wname, bname=None):
    y = xin @ W[wname].T
    if bname is not None and bname in W:
        y = y + W[bname]
    return y


# ---------------------------------------------------------------------------
# Definition: whole sequence
# ---------------------------------------------------------------------------
def forward_seq(cfg, W, ia3, x, dtype=np.float64):
    """ia3: {"k": l_k [nkv*d], "v": l_v [nkv*d], "ff": l_ff [F]}; every row carries the adapter."""
    W, ia3, x = _cast(W, dtype), _cast(ia3, dtype), np.asarray(x, dtype=dtype)
    n = x.shape[0]
    rows = np.ones(n, dtype=bool)
    pos = np.arange(n)
    h1 = ops.rmsnorm(x, W["g1"], cfg.rms_eps)
    q0 = _base(W, h1, "wq", "bq")
    k0 = _base(W, h1, "wk", "bk")
    v0 = _base(W, h1, "wv", "bv")
    k1 = bypass_scale(k0, ia3["k"], rows)
    v = bypass_scale(v0, ia3["v"], rows)
    q = ops.rope(q0, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta)
    k = ops.rope(k1, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta)
    a, lse = ops.attention(q, pos, k, v, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    x2 = x + _base(W, a, "wo")
    h2 = ops.rmsnorm(x2, W["g2"], cfg.rms_eps)
    gate, up = _base(W, h2, "wg"), _base(W, h2, "wu")
    act0 = ops.swiglu(gate, up)
    act = bypass_scale(act0, ia3["ff"], rows)
    y = x2 + _base(W, act, "wd")
    return dict(x=x, h1=h1, q=q, k0=k0, v0=v0, k=k, v=v, a=a, lse=lse, x2=x2, h2=h2, gate=gate, up=up,
                act0=act0, act=act, y=y)


def backward_seq(cfg, W, ia3, x, dY, dtype=np.float64):
    """Returns (dX, {"k": dl_k, "v": dl_v, "ff": dl_ff}, dK, dV); dK, dV w.r.t. the cached (scaled,
    rotated) keys and the cached values.  The frozen weights get no gradient (Sec. 5.2)."""
    W, ia3 = _cast(W, dtype), _cast(ia3, dtype)
    dY = np.asarray(dY, dtype=dtype)
    f = forward_seq(cfg, W, ia3, x, dtype)
    pos = np.arange(f["x"].shape[0])
    g = {}
    dact = dY @ W["wd"]                                   # w.r.t. the scaled activation
    g["ff"] = np.sum(dact * f["act0"], axis=0)
    dact0 = dact * ia3["ff"]
    dgate, dup = ops.swiglu_bwd(f["gate"], f["up"], dact0)
    dh2 = dgate @ W["wg"] + dup @ W["wu"]
    dx2 = dY + ops.rmsnorm_bwd(f["x2"], W["g2"], cfg.rms_eps, dh2)
    da = dx2 @ W["wo"]
    dq, dK, dV = ops.attention_bwd(f["q"], pos, f["k"], f["v"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, da)
    dq0 = ops.rope(dq, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta, inverse=True)
    dk1 = ops.rope(dK, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta, inverse=True)
    g["k"] = np.sum(dk1 * f["k0"], axis=0)
    g["v"] = np.sum(dV * f["v0"], axis=0)
    dh1 = dq0 @ W["wq"] + (dk1 * ia3["k"]) @ W["wk"] + (dV * ia3["v"]) @ W["wv"]
    dX = dx2 + ops.rmsnorm_bwd(f["x"], W["g1"], cfg.rms_eps, dh1)
    return dX, g, dK, dV


# ---------------------------------------------------------------------------
# Method: caches, windows, accumulator (Alg. 2)
# ---------------------------------------------------------------------------
def forward_mixed(cfg, W, ia3, maps, x, pool, ft_states=None, dtype=np.float64):
    """One forward iteration over a mixed token batch (Sec. 6.2).  Rows of requests with adapter >= 0 are
    scaled; finetune rows store Q and the pruned set in their Ia3FtState."""
    W, ia3, x = _cast(W, dtype), _cast(ia3, dtype), np.asarray(x, dtype=dtype)
    T = maps["T"]
    assert x.shape[0] == T
    rows = maps["tok_adapter"] >= 0
    pos = maps["tok_pos"]
    h1 = ops.rmsnorm(x, W["g1"], cfg.rms_eps)
    q0 = _base(W, h1, "wq", "bq")
    k0 = _base(W, h1, "wk", "bk")
    v0 = _base(W, h1, "wv", "bv")
    k1 = bypass_scale(k0, ia3["k"], rows)
    v = bypass_scale(v0, ia3["v"], rows)
    q = ops.rope(q0, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta)
    k = ops.rope(k1, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta)
    pool.k[maps["slot"]] = k
    pool.v[maps["slot"]] = v
    a, lse = attention_mixed(cfg, maps, q, pool)
    x2 = x + _base(W, a, "wo")
    h2 = ops.rmsnorm(x2, W["g2"], cfg.rms_eps)
    gate, up = _base(W, h2, "wg"), _base(W, h2, "wu")
    act = bypass_scale(ops.swiglu(gate, up), ia3["ff"], rows)
    y = x2 + _base(W, act, "wd")
    if ft_states is not None:
        for r in range(maps["n_req"]):
            if maps["req_kind"][r] != 2:
                continue
            st = ft_states[int(maps["req_seq"][r])]
            t0, t1 = maps["req_tok_off"][r], maps["req_tok_off"][r + 1]
            p = pos[t0:t1]
            st.q_cache[p] = q[t0:t1]
            st.x[p], st.x2[p] = x[t0:t1], x2[t0:t1]
            st.gate[p], st.up[p] = gate[t0:t1], up[t0:t1]
            st.k0[p], st.v0[p] = k0[t0:t1], v0[t0:t1]
            st.attn[p], st.lse[p] = a[t0:t1], lse[t0:t1]
    return y


def backward_window(cfg, W, ia3, st, K, V, win_start, win_len, dY, grads, need_dx=True, dtype=np.float64):
    """Backward of the token window [win_start, win_start + win_len) through the layer (Alg. 2's Backward,
    Add, Slice and CalculateGrads steps; Sec. 6.1).  K, V: the sequence's cached rows [0, l).  Windows are
    visited from the sequence end downwards.  The vectors' gradients are added into grads {"k", "v", "ff"}.
    Reads x, x2, gate, up, Q, K, V, k0, v0 from the state, nothing else."""
    W, ia3 = _cast(W, dtype), _cast(ia3, dtype)
    dY = np.asarray(dY, dtype=dtype)
    l = win_start + win_len
    w = slice(win_start, l)
    pos = np.arange(win_start, l)

    def add(name, val):
        grads[name] = grads[name] + val if name in grads else val

    x2 = st.x2[w]
    act0 = ops.swiglu(st.gate[w], st.up[w])               # rematerialised
    dact = dY @ W["wd"]
    add("ff", np.sum(dact * act0, axis=0))
    dgate, dup = ops.swiglu_bwd(st.gate[w], st.up[w], dact * ia3["ff"])
    dh2 = dgate @ W["wg"] + dup @ W["wu"]
    dx2 = dY + ops.rmsnorm_bwd(x2, W["g2"], cfg.rms_eps, dh2)
    da = dx2 @ W["wo"]
    dq, dK, dV = ops.attention_bwd(st.q_cache[w], pos, K[:l], V[:l], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, da)
    st.dk_accum[:l] += dK
    st.dv_accum[:l] += dV
    gk, gv = st.dk_accum[w], st.dv_accum[w]               # complete: every later query is done
    dk1 = ops.rope(gk, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta, inverse=True)
    add("k", np.sum(dk1 * st.k0[w], axis=0))
    add("v", np.sum(gv * st.v0[w], axis=0))
    if not need_dx:
        return None
    dq0 = ops.rope(dq, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta, inverse=True)
    dh1 = dq0 @ W["wq"] + (dk1 * ia3["k"]) @ W["wk"] + (gv * ia3["v"]) @ W["wv"]
    return dx2 + ops.rmsnorm_bwd(st.x[w], W["g1"], cfg.rms_eps, dh1)
