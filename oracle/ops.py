"""Per-operator definitions of the decoder layer (oracle side; test infrastructure).

The paper names its backbones (LLaMA-3.1, Qwen-2.5; Sec. 8) without restating their
operators; these are the textbook definitions of those families.  Row-vector
convention: activations are [tokens, features]; a base weight W is stored
[out_features, in_features], so a projection is  x @ W.T.  The LoRA bypass network
(Sec. 4.1,  Y = f_B(X) + f_A(X)) is  f_A(X) = scale * (X @ A) @ B  with
A [in, r], B [r, out].
"""
import numpy as np


# ---- RMSNorm --------------------------------------------------------------
def rmsnorm(x, g, eps):
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rmsnorm_bwd(x, g, eps, dh):
    """d/dx of  h = x * rstd * g,  rstd = (mean(x^2) + eps)^(-1/2)."""
    H = x.shape[-1]
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    gd = g * dh
    return rstd * gd - x * (rstd ** 3) * np.sum(x * gd, axis=-1, keepdims=True) / H


# ---- rotary position embedding -------------------------------------------
def rope(t, pos, n_heads, d, theta, inverse=False):
    """Rotate every head of t [n, n_heads*d] at absolute positions pos [n].
    Pair (i, i + d/2) of a head turns by the angle  pos * theta^(-2i/d).
    inverse=True turns by the negative angle (the transpose of the rotation,
    which is what the backward pass applies to a gradient)."""
    n = t.shape[0]
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    if inverse:
        ang = -ang
    c, s = np.cos(ang).astype(t.dtype), np.sin(ang).astype(t.dtype)
    th = t.reshape(n, n_heads, d)
    lo, hi = th[:, :, :half], th[:, :, half:]
    out = np.empty_like(th)
    out[:, :, :half] = lo * c[:, None, :] - hi * s[:, None, :]
    out[:, :, half:] = hi * c[:, None, :] + lo * s[:, None, :]
    return out.reshape(n, n_heads * d)


# ---- SwiGLU ---------------------------------------------------------------
def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def swiglu(gate, up):
    return gate * sigmoid(gate) * up


def swiglu_bwd(gate, up, dact):
    sg = sigmoid(gate)
    dgate = dact * up * (sg + gate * sg * (1.0 - sg))
    dup = dact * gate * sg
    return dgate, dup


# ---- causal attention over a cached prefix ---------------------------------
def attention(q, q_pos, K, V, n_q_heads, n_kv_heads, d):
    """Brute force.  q [n, nq*d] are queries at absolute positions q_pos [n]; K, V
    [m, nkv*d] are the (post-RoPE) keys and the values of positions 0..m-1 of the
    same sequence.  Query head h reads kv head h // (nq/nkv).  A query at position
    p sees positions 0..p (the causal rule of prefill, which finetuning tokens
    share: Sec. 6.2).  Returns (out [n, nq*d], lse [n, nq])."""
    n, m = q.shape[0], K.shape[0]
    group = n_q_heads // n_kv_heads
    q_pos = np.asarray(q_pos)
    visible = np.arange(m)[None, :] <= q_pos[:, None]          # [n, m]
    out = np.zeros_like(q)
    lse = np.zeros((n, n_q_heads), dtype=q.dtype)
    for h in range(n_q_heads):
        kh = h // group
        qh = q[:, h * d:(h + 1) * d]
        Kh = K[:, kh * d:(kh + 1) * d]
        Vh = V[:, kh * d:(kh + 1) * d]
        S = qh @ Kh.T / np.sqrt(d)
        S = np.where(visible, S, -np.inf)
        mx = S.max(axis=1, keepdims=True)
        E = np.exp(S - mx)
        Z = E.sum(axis=1, keepdims=True)
        P = E / Z
        out[:, h * d:(h + 1) * d] = P @ Vh
        lse[:, h] = (mx + np.log(Z))[:, 0]
    return out, lse


def attention_bwd(q, q_pos, K, V, n_q_heads, n_kv_heads, d, dout):
    """Gradients of attention() w.r.t. q [n, nq*d] and w.r.t. every cached row of
    K, V [m, nkv*d] (Sec. 6.1: dQ has the window's rows, dK/dV have all rows up to
    the window's end).  Softmax backward by its Jacobian:
    dS = P * (dP - rowsum(P * dP))."""
    n, m = q.shape[0], K.shape[0]
    group = n_q_heads // n_kv_heads
    q_pos = np.asarray(q_pos)
    visible = np.arange(m)[None, :] <= q_pos[:, None]
    dq = np.zeros_like(q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for h in range(n_q_heads):
        kh = h // group
        sl, ksl = slice(h * d, (h + 1) * d), slice(kh * d, (kh + 1) * d)
        S = q[:, sl] @ K[:, ksl].T / np.sqrt(d)
        S = np.where(visible, S, -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        P = E / E.sum(axis=1, keepdims=True)
        dO = dout[:, sl]
        dV[:, ksl] += P.T @ dO
        dP = dO @ V[:, ksl].T
        dS = P * (dP - np.sum(P * dP, axis=1, keepdims=True))
        dq[:, sl] = dS @ K[:, ksl] / np.sqrt(d)
        dK[:, ksl] += dS.T @ q[:, sl] / np.sqrt(d)
    return dq, dK, dV


# ---- LoRA bypass ------------------------------------------------------------
def lora_delta(x, A, B, scale):
    """f_A(X) = scale * (X A) B."""
    return scale * ((x @ A) @ B)


def lora_bwd(x, A, B, scale, dy):
    """For y = scale * (x A) B: returns (dx, dA, dB)."""
    t = dy @ B.T                  # [n, r]
    dB = scale * (x @ A).T @ dy
    dA = scale * x.T @ t
    dx = scale * t @ A.T
    return dx, dA, dB


# ---- storage types narrower than the arithmetic --------------------------------
def round_bf16(a):
    """Nearest bfloat16 value (8 significant bits, ties to even) of every element, returned in the
    input's own floating-point type.  Written from the format's definition: a = m * 2^e with
    0.5 <= |m| < 1, keep round_half_even(m * 2^8) / 2^8.  Values below the normal range of the format
    (|a| < 2^-126) are outside what the layer's tensors hold and are not treated specially."""
    a = np.asarray(a)
    m, e = np.frexp(a)
    return np.ldexp(np.rint(m * 256.0) / 256.0, e).astype(a.dtype)



# ---- ReLU with a sign bitmask (Sec. 5.2) -------------------------------------------------
def relu_bitmask_fwd(x):
    """y = max(x, 0) and the only thing its backward needs: one bit per element, "x > 0".  The bits of a row are
    packed into 32-bit words, bit j of word w = element 32 w + j (a convention; the paper fixes the idea - a
    bitmask in place of the tensor - not a layout); unused high bits of a row's last word are zero.
    Returns (y, mask [n, ceil(width / 32)] uint32)."""
    x = np.asarray(x)
    n, width = x.shape
    words = (width + 31) // 32
    pos = np.zeros((n, words * 32), dtype=np.uint64)
    pos[:, :width] = x > 0
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    mask = (pos.reshape(n, words, 32) * weights).sum(axis=2).astype(np.uint32)
    return np.maximum(x, 0), mask


def relu_bitmask_bwd(dy, mask):
    """dx = dy where the element's bit is set, 0 elsewhere."""
    dy = np.asarray(dy)
    n, width = dy.shape
    bits = (mask[:, :, None] >> np.arange(32, dtype=np.uint32)) & np.uint32(1)
    keep = bits.reshape(n, -1)[:, :width].astype(bool)
    return np.where(keep, dy, 0)
