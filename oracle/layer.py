"""One LoRA-augmented decoder layer: definition and the token-level method
(oracle side; test infrastructure).

Two ways to the same numbers:
  * the DEFINITION: whole-sequence forward and hand-derived backward of the layer
    (layer_forward_seq / layer_backward_seq).  Frozen base weights receive no
    gradient (Sec. 5.2); only LoRA matrices and the layer input do.
  * the METHOD: Algorithm 2.  Forward over token windows against cached K/V
    (layer_forward_mixed, which also serves decode tokens and prefill chunks of the
    same batch, Sec. 6.2), then backward over windows from the sequence end with a
    KV-gradient accumulator (layer_backward_window; Sec. 6.1 and Sec. 7), reading
    only the activations graph pruning keeps (Algorithm 1): x, x2, gate, up, Q, K, V
    (and the attention output when the output projection carries LoRA).

Storage rounding (optional, `storage=` of the METHOD's two functions): the paper says nothing
about where a reduced-precision run rounds.  Reading: a configuration whose storage type is
narrower than the arithmetic rounds every tensor it WRITES TO MEMORY (norm outputs, projection
outputs, rotated q / k and the cached K / V / Q rows, attention output, x2, gate, up, their
product, y; in the backward pass every gradient handed from one operator to the next) and
nothing else; accumulators (LoRA gradients, KV-gradient accumulator, log-sum-exp) stay wide.
`storage` names that rounding ("bf16", or a function array -> array; None = no rounding, the
default and the definition); all arithmetic stays in `dtype`.  It exists to tell apart, in a parity test,
error that comes from the storage type itself from error of the arithmetic under test.

Readings of Algorithm 2 taken here: the position update l_{j+1} = l_j - s_j belongs
inside the window loop; "Add" means accum[0:l_j) += (dK, dV); in the backward pass
l_j is the exclusive END of window j and Slice takes the s_j rows ending there.
"""
import numpy as np

from . import ops

TARGETS = ("q", "k", "v", "o", "gate", "up", "down")


def _cast(tree, dtype):
    if isinstance(tree, dict):
        return {k: _cast(v, dtype) for k, v in tree.items()}
    if isinstance(tree, (tuple, list)):
        return type(tree)(_cast(v, dtype) for v in tree)
    return np.asarray(tree, dtype=dtype)


def _proj(cfg, W, lora, target, wname, bname, xin, lora_rows):
    """Base projection plus the bypass network on the rows that carry an adapter.
    lora / lora_rows: one adapter and its row mask, or lists of both (several adapters in one
    batch, each on its own rows)."""
    y = xin @ W[wname].T
    if bname is not None and bname in W:
        y = y + W[bname]
    pairs = zip(lora, lora_rows) if isinstance(lora, list) else [(lora, lora_rows)]
    for lo, rows in pairs:
        if lo is not None and target in lo and rows is not None and np.any(rows):
            A, B = lo[target]
            y = y.copy()
            y[rows] += ops.lora_delta(xin[rows], A, B, cfg.lora_scale)
    return y


# ---------------------------------------------------------------------------
# Definition: whole sequence
# ---------------------------------------------------------------------------
def layer_forward_seq(cfg, W, lora, x, dtype=np.float64):
    """Forward of positions 0..n-1 of one sequence, all rows carrying the adapter
    (lora=None: base model).  Returns every intermediate by name."""
    W, lora, x = _cast(W, dtype), (_cast(lora, dtype) if lora else None), np.asarray(x, dtype=dtype)
    n = x.shape[0]
    rows = np.ones(n, dtype=bool)
    pos = np.arange(n)
    h1 = ops.rmsnorm(x, W["g1"], cfg.rms_eps)
    q0 = _proj(cfg, W, lora, "q", "wq", "bq", h1, rows)
    k0 = _proj(cfg, W, lora, "k", "wk", "bk", h1, rows)
    v = _proj(cfg, W, lora, "v", "wv", "bv", h1, rows)
    q = ops.rope(q0, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta)
    k = ops.rope(k0, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta)
    a, lse = ops.attention(q, pos, k, v, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    x2 = x + _proj(cfg, W, lora, "o", "wo", None, a, rows)
    h2 = ops.rmsnorm(x2, W["g2"], cfg.rms_eps)
    gate = _proj(cfg, W, lora, "gate", "wg", None, h2, rows)
    up = _proj(cfg, W, lora, "up", "wu", None, h2, rows)
    act = ops.swiglu(gate, up)
    y = x2 + _proj(cfg, W, lora, "down", "wd", None, act, rows)
    return dict(x=x, h1=h1, q=q, k=k, v=v, a=a, lse=lse, x2=x2, h2=h2, gate=gate, up=up,
                act=act, y=y)


def _proj_bwd(cfg, W, lora, target, wname, xin, dy, grads):
    """Input gradient of a projection; adds the LoRA matrices' gradients to grads.
    The base weight gets none (it is frozen)."""
    dx = dy @ W[wname]
    if lora is not None and target in lora:
        A, B = lora[target]
        dxl, dA, dB = ops.lora_bwd(xin, A, B, cfg.lora_scale, dy)
        dx = dx + dxl
        if target in grads:
            grads[target] = (grads[target][0] + dA, grads[target][1] + dB)
        else:
            grads[target] = (dA, dB)
    return dx


def layer_backward_seq(cfg, W, lora, x, dY, dtype=np.float64):
    """Whole-sequence backward.  Returns (dX, grads {target: (dA, dB)}, dK, dV) where
    dK, dV are the gradients w.r.t. the post-RoPE keys and the values."""
    W, lora = _cast(W, dtype), _cast(lora, dtype)
    dY = np.asarray(dY, dtype=dtype)
    f = layer_forward_seq(cfg, W, lora, x, dtype)
    n = f["x"].shape[0]
    pos = np.arange(n)
    grads = {}
    dact = _proj_bwd(cfg, W, lora, "down", "wd", f["act"], dY, grads)
    dgate, dup = ops.swiglu_bwd(f["gate"], f["up"], dact)
    dh2 = _proj_bwd(cfg, W, lora, "gate", "wg", f["h2"], dgate, grads) \
        + _proj_bwd(cfg, W, lora, "up", "wu", f["h2"], dup, grads)
    dx2 = dY + ops.rmsnorm_bwd(f["x2"], W["g2"], cfg.rms_eps, dh2)
    da = _proj_bwd(cfg, W, lora, "o", "wo", f["a"], dx2, grads)
    dq, dK, dV = ops.attention_bwd(f["q"], pos, f["k"], f["v"], cfg.n_q_heads, cfg.n_kv_heads,
                                   cfg.head_dim, da)
    dq0 = ops.rope(dq, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta, inverse=True)
    dk0 = ops.rope(dK, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta, inverse=True)
    dh1 = _proj_bwd(cfg, W, lora, "q", "wq", f["h1"], dq0, grads) \
        + _proj_bwd(cfg, W, lora, "k", "wk", f["h1"], dk0, grads) \
        + _proj_bwd(cfg, W, lora, "v", "wv", f["h1"], dV, grads)
    dX = dx2 + ops.rmsnorm_bwd(f["x"], W["g1"], cfg.rms_eps, dh1)
    return dX, grads, dK, dV


# ---------------------------------------------------------------------------
# Method: caches, windows, accumulator
# ---------------------------------------------------------------------------
class KVPool:
    """Paged cache: slot-indexed rows (slot = page * page_size + offset)."""

    def __init__(self, num_pages, page_size, kv_dim, dtype=np.float64):
        self.page_size = page_size
        self.k = np.zeros((num_pages * page_size, kv_dim), dtype=dtype)
        self.v = np.zeros((num_pages * page_size, kv_dim), dtype=dtype)

    def slots(self, pages, n):
        p = np.arange(n)
        return np.asarray(pages)[p // self.page_size].astype(np.int64) * self.page_size + p % self.page_size


class FtState:
    """Per-layer state of one finetune sequence of length L: the Q cache of Alg. 2
    (K, V live in the paged pool like any other sequence's), the activations kept
    by pruning, and the statically allocated KV-gradient accumulator (Sec. 7)."""

    def __init__(self, cfg, L, dtype=np.float64):
        self.L = L
        z = lambda w: np.zeros((L, w), dtype=dtype)
        self.q_cache = z(cfg.q_dim)
        self.x, self.x2 = z(cfg.hidden), z(cfg.hidden)
        self.gate, self.up = z(cfg.ffn), z(cfg.ffn)
        self.attn = z(cfg.q_dim)
        self.lse = z(cfg.n_q_heads)
        self.dk_accum, self.dv_accum = z(cfg.kv_dim), z(cfg.kv_dim)


def _storage_fn(storage, dtype):
    """storage: None (no rounding), "bf16", or a function array -> array"""
    if storage is None:
        return lambda a: a
    if storage == "bf16":
        return lambda a: ops.round_bf16(np.asarray(a, dtype=dtype))
    return lambda a: np.asarray(storage(a), dtype=dtype)


def layer_forward_mixed(cfg, W, lora, maps, x, pool, ft_states=None, dtype=np.float64,
                        return_all=False, storage=None):
    """One forward iteration of the layer over a mixed token batch, through the
    caches.  maps: oracle.maps.build_maps output.  pool: KVPool (new K/V rows are
    appended at the tokens' slots).  ft_states: {seq_id: FtState}; rows of finetune
    windows store Q and the pruned activation set there.  lora: one adapter {target: (A, B)},
    applied to the rows whose segment has adapter >= 0; or, with several adapters served in one
    batch (Sec. 6.2: the inference requests of a batch may belong to different PEFT models), a
    list of adapters indexed by adapter id, each applied to the rows of its own requests.
    storage: rounding applied to every tensor written to memory (see the module header)."""
    W, x = _cast(W, dtype), np.asarray(x, dtype=dtype)
    sr = _storage_fn(storage, dtype)
    T = maps["T"]
    assert x.shape[0] == T
    if isinstance(lora, list):
        lora = [_cast(lo, dtype) if lo else None for lo in lora]
        assert int(maps["tok_adapter"].max()) < len(lora)
        rows = [maps["tok_adapter"] == a for a in range(len(lora))]
    else:
        lora = _cast(lora, dtype) if lora else None
        rows = np.zeros(T, dtype=bool)
        for s in range(maps["n_seg"]):
            if maps["seg_adapter"][s] >= 0:
                rows[maps["seg_off"][s]:maps["seg_off"][s + 1]] = True
    pos = maps["tok_pos"]
    h1 = sr(ops.rmsnorm(x, W["g1"], cfg.rms_eps))
    q0 = sr(_proj(cfg, W, lora, "q", "wq", "bq", h1, rows))
    k0 = sr(_proj(cfg, W, lora, "k", "wk", "bk", h1, rows))
    v = sr(_proj(cfg, W, lora, "v", "wv", "bv", h1, rows))
    q = sr(ops.rope(q0, pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta))
    k = sr(ops.rope(k0, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta))
    pool.k[maps["slot"]] = k
    pool.v[maps["slot"]] = v
    a, lse = attention_mixed(cfg, maps, q, pool)
    a = sr(a)
    x2 = sr(x + _proj(cfg, W, lora, "o", "wo", None, a, rows))
    h2 = sr(ops.rmsnorm(x2, W["g2"], cfg.rms_eps))
    gate = sr(_proj(cfg, W, lora, "gate", "wg", None, h2, rows))
    up = sr(_proj(cfg, W, lora, "up", "wu", None, h2, rows))
    act = sr(ops.swiglu(gate, up))
    y = sr(x2 + _proj(cfg, W, lora, "down", "wd", None, act, rows))
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
            st.attn[p], st.lse[p] = a[t0:t1], lse[t0:t1]
    if return_all:
        return dict(h1=h1, q=q, k=k, v=v, a=a, lse=lse, x2=x2, h2=h2, gate=gate, up=up, act=act, y=y)
    return y


def attention_mixed(cfg, maps, q, pool):
    """Attention of every token of the batch against its own sequence's cached
    positions 0..pos, read through the block table."""
    T = maps["T"]
    ps = maps["page_size"]
    a = np.zeros((T, cfg.q_dim), dtype=q.dtype)
    lse = np.zeros((T, cfg.n_q_heads), dtype=q.dtype)
    for r in range(maps["n_req"]):
        t0, t1 = maps["req_tok_off"][r], maps["req_tok_off"][r + 1]
        kv_len = int(maps["req_kv_len"][r])
        p = np.arange(kv_len)
        slots = maps["block_table"][r][p // ps].astype(np.int64) * ps + p % ps
        a[t0:t1], lse[t0:t1] = ops.attention(q[t0:t1], maps["tok_pos"][t0:t1], pool.k[slots],
                                             pool.v[slots], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    return a, lse


def layer_backward_window(cfg, W, lora, st, K, V, win_start, win_len, dY, grads, need_dx=True,
                          dtype=np.float64, storage=None):
    """Backward of one token window [win_start, win_start + win_len) of a finetune
    sequence through one layer (Alg. 2, the Backward / Add / Slice / CalculateGrads
    steps).  st: FtState filled by the forward windows.  K, V: the sequence's cached
    rows [0, l) with l = win_start + win_len (every earlier position, Sec. 6.1).
    Windows must be visited from the sequence end downwards, so that when a window
    runs, st.dk_accum / st.dv_accum already hold the contributions of all later
    queries and its own rows become complete.  LoRA gradients are added into grads
    {target: (dA, dB)}.  Returns dX [win_len, H] (None when need_dx is False: no
    trainable parameter below, Alg. 1's dead-output propagation).
    Reads only x, x2, gate, up, Q, K, V (+ attn if 'o' carries LoRA) from the state.
    storage: rounding applied to every rematerialised activation and every gradient handed from
    one operator to the next (see the module header); the accumulators are not rounded."""
    W, lora = _cast(W, dtype), _cast(lora, dtype)
    sr = _storage_fn(storage, dtype)
    dY = np.asarray(dY, dtype=dtype)
    l = win_start + win_len
    w = slice(win_start, l)
    pos = np.arange(win_start, l)
    # --- MLP side (row-local); h2 and act are rematerialized --------------------
    x2 = st.x2[w]
    h2 = sr(ops.rmsnorm(x2, W["g2"], cfg.rms_eps))
    act = sr(ops.swiglu(st.gate[w], st.up[w]))
    dact = sr(_proj_bwd(cfg, W, lora, "down", "wd", act, dY, grads))
    dgate, dup = ops.swiglu_bwd(st.gate[w], st.up[w], dact)
    dgate, dup = sr(dgate), sr(dup)
    dh2 = sr(_proj_bwd(cfg, W, lora, "gate", "wg", h2, dgate, grads)
             + _proj_bwd(cfg, W, lora, "up", "wu", h2, dup, grads))
    dx2 = sr(dY + ops.rmsnorm_bwd(x2, W["g2"], cfg.rms_eps, dh2))
    attn_in = st.attn[w] if (lora and "o" in lora) else np.zeros((win_len, cfg.q_dim), dtype=dtype)
    da = sr(_proj_bwd(cfg, W, lora, "o", "wo", attn_in, dx2, grads))
    # --- attention: dQ for the window, dK/dV for every row before its end ------
    dq, dK, dV = ops.attention_bwd(st.q_cache[w], pos, K[:l], V[:l], cfg.n_q_heads, cfg.n_kv_heads,
                                   cfg.head_dim, da)
    st.dk_accum[:l] += dK
    st.dv_accum[:l] += dV
    gk, gv = st.dk_accum[w], st.dv_accum[w]          # complete: all later queries are done
    # --- q/k/v side -------------------------------------------------------------
    if not need_dx and not any(t in lora for t in ("q", "k", "v")):
        return None
    x = st.x[w]
    h1 = sr(ops.rmsnorm(x, W["g1"], cfg.rms_eps))
    dq0 = sr(ops.rope(sr(dq), pos, cfg.n_q_heads, cfg.head_dim, cfg.rope_theta, inverse=True))
    dk0 = sr(ops.rope(gk, pos, cfg.n_kv_heads, cfg.head_dim, cfg.rope_theta, inverse=True))
    dh1 = sr(_proj_bwd(cfg, W, lora, "q", "wq", h1, dq0, grads)
             + _proj_bwd(cfg, W, lora, "k", "wk", h1, dk0, grads)
             + _proj_bwd(cfg, W, lora, "v", "wv", h1, sr(gv), grads))
    if not need_dx:
        return None
    return sr(dx2 + ops.rmsnorm_bwd(x, W["g1"], cfg.rms_eps, dh1))


# ---------------------------------------------------------------------------
# Drivers over a stack of layers
# ---------------------------------------------------------------------------
def mse_loss_grad(y, target):
    """loss = mean over all L*H elements of (y - target)^2; returns (loss, dloss/dy).
    Normalising by the whole sequence makes the loss independent of the windows."""
    diff = y - target
    return float(np.mean(diff * diff)), 2.0 * diff / diff.size


def finetune_whole_seq(cfg, layers, loras, x, target, dtype=np.float64):
    """Sequence-level finetuning step of a stack of layers: forward all, MSE loss on
    the top output, backward all.  Returns (loss, [grads per layer], dX0)."""
    x = np.asarray(x, dtype=dtype)
    inputs = []
    h = x
    for W, lo in zip(layers, loras):
        inputs.append(h)
        h = layer_forward_seq(cfg, W, lo, h, dtype)["y"]
    loss, dY = mse_loss_grad(h, np.asarray(target, dtype=dtype))
    all_grads = [None] * len(layers)
    for n in range(len(layers) - 1, -1, -1):
        dY, g, _, _ = layer_backward_seq(cfg, layers[n], loras[n], inputs[n], dY, dtype)
        all_grads[n] = g
    return loss, all_grads, dY


def finetune_token_level(cfg, layers, loras, x, target, fwd_windows, bwd_windows, page_size=16,
                         dtype=np.float64, pages=None):
    """Algorithm 2 for one finetune sequence alone in the batch.  fwd_windows /
    bwd_windows: window lengths (each list sums to L); forward windows run from the
    sequence start, backward windows from its end.  Returns (loss, grads, dX0)."""
    from .maps import build_maps
    from types import SimpleNamespace as NS
    x = np.asarray(x, dtype=dtype)
    target = np.asarray(target, dtype=dtype)
    L, N = x.shape[0], len(layers)
    assert sum(fwd_windows) == L and sum(bwd_windows) == L
    n_pages = -(-L // page_size)
    pages = np.arange(n_pages) if pages is None else np.asarray(pages)
    pools = [KVPool(int(pages.max()) + 1, page_size, cfg.kv_dim, dtype) for _ in range(N)]
    states = [FtState(cfg, L, dtype) for _ in range(N)]
    Y = np.zeros((L, cfg.hidden), dtype=dtype)
    l = 0
    for s in fwd_windows:                                   # forward pass
        maps = build_maps([NS(kind=2, seq_id=0, start_pos=l, n_new=s, adapter=0)], {0: pages}, page_size)
        h = x[l:l + s]
        for n in range(N):
            h = layer_forward_mixed(cfg, layers[n], loras[n], maps, h, pools[n], {0: states[n]}, dtype)
        Y[l:l + s] = h
        l += s
    loss, dYtop = mse_loss_grad(Y, target)
    grads = [dict() for _ in range(N)]
    dcur = dYtop
    slots = pools[0].slots(pages, L)
    for n in range(N - 1, -1, -1):                          # backward pass, layer by layer
        dnext = np.zeros_like(dcur)
        l = L
        for s in bwd_windows:                               # windows from the end
            K, V = pools[n].k[slots[:l]], pools[n].v[slots[:l]]
            dnext[l - s:l] = layer_backward_window(cfg, layers[n], loras[n], states[n], K, V, l - s, s,
                                                   dcur[l - s:l], grads[n], True, dtype)
            l -= s
        dcur = dnext
    return loss, grads, dcur, states
