"""Pins for oracle/ops.py: closed forms, library routines, finite differences.
None of the expected values below comes from the function under test."""
import math

import numpy as np
import pytest
import scipy.special
import torch
import torch.nn.functional as F

from oracle import ops
from helpers import rel_err

RNG = np.random.default_rng(7)


def fd_check(f, x, dx_analytic, n_samples=12, h=1e-6, tol=1e-6, rng=RNG):
    """central finite differences of scalar f at sampled elements of x"""
    flat = x.reshape(-1)
    idx = rng.choice(flat.size, size=min(n_samples, flat.size), replace=False)
    for i in idx:
        old = flat[i]
        flat[i] = old + h
        fp = f()
        flat[i] = old - h
        fm = f()
        flat[i] = old
        num = (fp - fm) / (2 * h)
        ana = dx_analytic.reshape(-1)[i]
        assert abs(num - ana) <= tol * max(1.0, abs(num), abs(ana)), (i, num, ana)


# ---- RMSNorm ----------------------------------------------------------------
def test_rmsnorm_unit_rms_and_scale_invariance():
    x = RNG.standard_normal((5, 16))
    h = ops.rmsnorm(x, np.ones(16), 0.0)
    assert np.allclose(np.sqrt(np.mean(h * h, axis=-1)), 1.0, atol=1e-12)
    assert np.allclose(ops.rmsnorm(3.7 * x, np.ones(16), 0.0), h, atol=1e-12)


def test_rmsnorm_hand_value():
    # x = (3, 4): mean square 12.5; eps 0.5 -> rstd = 1/sqrt(13); gains (2, -1)
    h = ops.rmsnorm(np.array([[3.0, 4.0]]), np.array([2.0, -1.0]), 0.5)
    assert np.allclose(h, [[6.0 / math.sqrt(13.0), -4.0 / math.sqrt(13.0)]], atol=1e-14)


def test_rmsnorm_matches_library():
    x, g = RNG.standard_normal((6, 24)), RNG.standard_normal(24)
    ref = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(ops.rmsnorm(x, g, 1e-5), ref, atol=1e-12)


def test_rmsnorm_bwd_fd():
    x, g, dh = RNG.standard_normal((3, 10)), RNG.standard_normal(10), RNG.standard_normal((3, 10))
    dx = ops.rmsnorm_bwd(x, g, 1e-5, dh)
    fd_check(lambda: float(np.sum(ops.rmsnorm(x, g, 1e-5) * dh)), x, dx)


# ---- RoPE -------------------------------------------------------------------
def test_rope_hand_value():
    # one head, d = 4, theta = 10000, position 3: pair (0,2) turns by 3 rad,
    # pair (1,3) by 3 * 10000^(-2/4) = 0.03 rad
    t = np.array([[1.0, 2.0, 3.0, 4.0]])
    out = ops.rope(t, [3], 1, 4, 10000.0)
    c0, s0, c1, s1 = math.cos(3.0), math.sin(3.0), math.cos(0.03), math.sin(0.03)
    exp = [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 3 * c0 + 1 * s0, 4 * c1 + 2 * s1]
    assert np.allclose(out[0], exp, atol=1e-14)


def test_rope_identity_norm_inverse_relative():
    nh, d = 3, 8
    t = RNG.standard_normal((5, nh * d))
    pos = np.array([0, 1, 7, 100, 4095])
    r = ops.rope(t, pos, nh, d, 500000.0)
    assert np.array_equal(r[0], t[0])                                  # position 0: identity
    assert np.allclose(np.linalg.norm(r.reshape(5, nh, d), axis=-1),
                       np.linalg.norm(t.reshape(5, nh, d), axis=-1), atol=1e-12)
    assert np.allclose(ops.rope(r, pos, nh, d, 500000.0, inverse=True), t, atol=1e-12)
    # scores depend on the position difference only
    q, k = RNG.standard_normal((1, d)), RNG.standard_normal((1, d))
    s1 = ops.rope(q, [10], 1, d, 1e4) @ ops.rope(k, [3], 1, d, 1e4).T
    s2 = ops.rope(q, [1010], 1, d, 1e4) @ ops.rope(k, [1003], 1, d, 1e4).T
    assert np.allclose(s1, s2, atol=1e-10)


def test_rope_backward_is_transpose():
    nh, d = 2, 8
    t, g = RNG.standard_normal((4, nh * d)), RNG.standard_normal((4, nh * d))
    pos = np.array([2, 3, 9, 31])
    lhs = np.sum(ops.rope(t, pos, nh, d, 1e4) * g)
    rhs = np.sum(t * ops.rope(g, pos, nh, d, 1e4, inverse=True))
    assert abs(lhs - rhs) < 1e-12


# ---- SwiGLU -----------------------------------------------------------------
def test_swiglu_values_and_library():
    assert ops.swiglu(np.array([0.0]), np.array([5.0]))[0] == 0.0
    assert abs(ops.swiglu(np.array([1.0]), np.array([2.0]))[0] - 2.0 / (1.0 + math.exp(-1.0))) < 1e-15
    g, u = RNG.standard_normal((4, 9)), RNG.standard_normal((4, 9))
    ref = (F.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    assert np.allclose(ops.swiglu(g, u), ref, atol=1e-14)


def test_swiglu_bwd_fd():
    g, u, da = RNG.standard_normal((3, 7)), RNG.standard_normal((3, 7)), RNG.standard_normal((3, 7))
    dg, du = ops.swiglu_bwd(g, u, da)
    fd_check(lambda: float(np.sum(ops.swiglu(g, u) * da)), g, dg)
    fd_check(lambda: float(np.sum(ops.swiglu(g, u) * da)), u, du)


# ---- attention --------------------------------------------------------------
def brute_attention(q, q_pos, K, V, nq, nkv, d):
    """token-by-token, head-by-head, with scipy's softmax"""
    out = np.zeros_like(q)
    for i in range(q.shape[0]):
        for h in range(nq):
            kh = h // (nq // nkv)
            n_vis = q_pos[i] + 1
            s = np.array([np.dot(q[i, h * d:(h + 1) * d], K[j, kh * d:(kh + 1) * d]) / math.sqrt(d)
                          for j in range(n_vis)])
            p = scipy.special.softmax(s)
            for j in range(n_vis):
                out[i, h * d:(h + 1) * d] += p[j] * V[j, kh * d:(kh + 1) * d]
    return out


@pytest.mark.parametrize("nq,nkv", [(4, 4), (4, 2), (6, 1)])
def test_attention_bruteforce(nq, nkv):
    d, m = 8, 13
    K, V = RNG.standard_normal((m, nkv * d)), RNG.standard_normal((m, nkv * d))
    q_pos = np.array([0, 5, 12, 12, 7])
    q = RNG.standard_normal((5, nq * d))
    out, lse = ops.attention(q, q_pos, K, V, nq, nkv, d)
    assert np.allclose(out, brute_attention(q, q_pos, K, V, nq, nkv, d), atol=1e-12)
    # lse against scipy
    for i in (1, 4):
        for h in range(nq):
            kh = h // (nq // nkv)
            s = q[i, h * d:(h + 1) * d] @ K[:q_pos[i] + 1, kh * d:(kh + 1) * d].T / math.sqrt(d)
            assert abs(lse[i, h] - scipy.special.logsumexp(s)) < 1e-12


def test_attention_properties():
    nq, nkv, d, m = 4, 2, 8, 9
    K, V = RNG.standard_normal((m, nkv * d)), RNG.standard_normal((m, nkv * d))
    q = RNG.standard_normal((3, nq * d))
    pos = np.array([0, 4, 8])
    out, _ = ops.attention(q, pos, K, V, nq, nkv, d)
    # a single visible key returns that key's value
    assert np.allclose(out[0].reshape(nq, d), np.repeat(V[0].reshape(nkv, d), nq // nkv, axis=0), atol=1e-14)
    # probabilities sum to one: constant values come back unchanged
    ones, _ = ops.attention(q, pos, K, np.ones_like(V), nq, nkv, d)
    assert np.allclose(ones, 1.0, atol=1e-13)
    # zero queries: uniform average of the visible values
    avg, _ = ops.attention(np.zeros_like(q), pos, K, V, nq, nkv, d)
    assert np.allclose(avg[1].reshape(nq, d)[0], V[:5, :d].mean(axis=0), atol=1e-13)
    # adding one vector to every key shifts each row of scores by a constant
    shifted, _ = ops.attention(q, pos, K + RNG.standard_normal((1, nkv * d)), V, nq, nkv, d)
    assert np.allclose(shifted, out, atol=1e-12)
    # grouped-query attention == multi-head attention on explicitly repeated kv heads
    rep = lambda t: np.repeat(t.reshape(m, nkv, d), nq // nkv, axis=1).reshape(m, nq * d)
    mha, _ = ops.attention(q, pos, rep(K), rep(V), nq, nq, d)
    assert np.allclose(mha, out, atol=1e-13)


def test_attention_matches_library_sdpa_and_autograd():
    nq, nkv, d, m, n = 4, 2, 8, 11, 6
    K, V = RNG.standard_normal((m, nkv * d)), RNG.standard_normal((m, nkv * d))
    q = RNG.standard_normal((n, nq * d))
    pos = np.arange(m - n, m)
    dout = RNG.standard_normal((n, nq * d))
    tq = torch.from_numpy(q).reshape(n, nq, d).transpose(0, 1).unsqueeze(0).requires_grad_()
    tk = torch.from_numpy(K).reshape(m, nkv, d).transpose(0, 1).unsqueeze(0).requires_grad_()
    tv = torch.from_numpy(V).reshape(m, nkv, d).transpose(0, 1).unsqueeze(0).requires_grad_()
    mask = torch.from_numpy(np.arange(m)[None, :] <= pos[:, None])
    ref = F.scaled_dot_product_attention(tq, tk.repeat_interleave(nq // nkv, 1), tv.repeat_interleave(nq // nkv, 1),
                                         attn_mask=mask)
    ref2 = ref[0].transpose(0, 1).reshape(n, nq * d)
    out, _ = ops.attention(q, pos, K, V, nq, nkv, d)
    assert np.allclose(out, ref2.detach().numpy(), atol=1e-12)
    ref2.backward(torch.from_numpy(dout))
    dq, dK, dV = ops.attention_bwd(q, pos, K, V, nq, nkv, d, dout)
    assert np.allclose(dq, tq.grad[0].transpose(0, 1).reshape(n, nq * d).numpy(), atol=1e-12)
    assert np.allclose(dK, tk.grad[0].transpose(0, 1).reshape(m, nkv * d).numpy(), atol=1e-12)
    assert np.allclose(dV, tv.grad[0].transpose(0, 1).reshape(m, nkv * d).numpy(), atol=1e-12)


def test_attention_bwd_fd():
    nq, nkv, d, m = 4, 2, 4, 7
    K, V = RNG.standard_normal((m, nkv * d)), RNG.standard_normal((m, nkv * d))
    q, pos = RNG.standard_normal((3, nq * d)), np.array([2, 5, 6])
    dout = RNG.standard_normal((3, nq * d))
    dq, dK, dV = ops.attention_bwd(q, pos, K, V, nq, nkv, d, dout)
    f = lambda: float(np.sum(ops.attention(q, pos, K, V, nq, nkv, d)[0] * dout))
    fd_check(f, q, dq)
    fd_check(f, K, dK)
    fd_check(f, V, dV)
    assert np.all(dK[pos.max() + 1:] == 0)     # no query sees later positions


# ---- LoRA -------------------------------------------------------------------
def test_lora_delta_orientation_and_scale():
    # x [1,2], A [2,1], B [1,3]: (x A) = 1*2 + 2*3 = 8; times B = (8, -8, 4); scale 0.5
    x, A, B = np.array([[1.0, 2.0]]), np.array([[2.0], [3.0]]), np.array([[1.0, -1.0, 0.5]])
    assert np.array_equal(ops.lora_delta(x, A, B, 0.5), [[4.0, -4.0, 2.0]])


def test_lora_bwd_fd():
    x, A, B = RNG.standard_normal((5, 6)), RNG.standard_normal((6, 2)), RNG.standard_normal((2, 4))
    dy = RNG.standard_normal((5, 4))
    dx, dA, dB = ops.lora_bwd(x, A, B, 1.7, dy)
    f = lambda: float(np.sum(ops.lora_delta(x, A, B, 1.7) * dy))
    fd_check(f, x, dx)
    fd_check(f, A, dA)
    fd_check(f, B, dB)


# ---- ReLU sign bitmask (Sec. 5.2) ------------------------------------------------------------
def test_relu_bitmask_hand_case_and_size():
    from oracle import ops
    x = np.zeros((2, 40))
    x[0, [0, 3, 31, 32, 39]] = [1.0, 0.5, 2.0, 7.0, 1e-30]
    x[0, [1, 2]] = [-1.0, -0.0]
    x[1, :] = -1.0
    x[1, 33] = 3.0
    y, m = ops.relu_bitmask_fwd(x)
    assert m.dtype == np.uint32 and m.shape == (2, 2)                 # 1 bit per element, rows padded to whole words
    assert m[0, 0] == (1 << 0) | (1 << 3) | (1 << 31) and m[0, 1] == (1 << 0) | (1 << 7)
    assert m[1, 0] == 0 and m[1, 1] == (1 << 1)
    assert np.array_equal(y, np.maximum(x, 0))


def test_relu_bitmask_backward_is_the_relu_jacobian():
    """dx from the bitmask alone equals the gradient of sum(relu(x) * dy) by the definition (and by library autograd)"""
    from oracle import ops
    import torch
    g = np.random.default_rng(5)
    for width in (1, 31, 32, 33, 70, 128):
        x, dy = g.standard_normal((7, width)), g.standard_normal((7, width))
        x[g.random((7, width)) < 0.1] = 0.0                             # exact zeros: the gradient there is 0
        _, m = ops.relu_bitmask_fwd(x)
        dx = ops.relu_bitmask_bwd(dy, m)
        assert np.array_equal(dx, dy * (x > 0))
        xt = torch.tensor(x, requires_grad=True)
        (torch.relu(xt) * torch.tensor(dy)).sum().backward()
        assert np.array_equal(dx, xt.grad.numpy())
        # the unused bits of the last word are zero
        if width % 32:
            assert np.all(m[:, -1] >> np.uint32(width % 32) == 0)
