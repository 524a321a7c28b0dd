"""Pins for oracle/ia3.py, the decoder layer with an (IA)^3 bypass network (Sec. 4.1): vectors of ones
give the base layer bit for bit; the scaled layer equals the BASE layer with the scales folded into
the frozen weights (an independent route through oracle/layer.py and, for the gradients, through
library autograd); gradients equal central finite differences; Algorithm 2's windows equal the whole
sequence; rows without the adapter do not see it; what the window backward reads is what graph
pruning (Alg. 1) keeps."""
from types import SimpleNamespace as NS

import numpy as np
import pytest
import torch

from oracle import ia3 as I
from oracle import layer as L
from oracle import prune as P
from oracle.maps import build_maps
from workload import gen
from helpers import SMALL, small_layer, rel_err
from test_oracle_layer import torch_layer

RNG = np.random.default_rng(23)
CFG = SMALL.with_(lora_targets=())


def setup(n=10, seed=5):
    W, _ = small_layer(SMALL)
    ia3 = {k: v.astype(np.float64) for k, v in gen.ia3_weights(CFG, seed).items()}
    x = gen.rng(seed, "ia3x", n).standard_normal((n, CFG.hidden))
    return W, ia3, x


def folded(W, ia3):
    """The base weights with the three vectors multiplied in: rows of Wk, Wv (and their biases), columns of Wd."""
    Wf = dict(W)
    Wf["wk"], Wf["wv"] = W["wk"] * ia3["k"][:, None], W["wv"] * ia3["v"][:, None]
    if "bk" in W:
        Wf["bk"], Wf["bv"] = W["bk"] * ia3["k"], W["bv"] * ia3["v"]
    Wf["wd"] = W["wd"] * ia3["ff"][None, :]
    return Wf


def test_vectors_of_ones_are_the_base_layer_bit_for_bit():
    W, ia3, x = setup()
    ones = {k: np.ones_like(v) for k, v in ia3.items()}
    base = L.layer_forward_seq(CFG, W, None, x)
    got = I.forward_seq(CFG, W, ones, x)
    for name in ("y", "k", "v", "a", "x2"):
        assert np.array_equal(got[name], base[name]), name
    assert not np.array_equal(I.forward_seq(CFG, W, ia3, x)["y"], base["y"])


def test_bypass_form_is_the_elementwise_product():
    t = RNG.standard_normal((6, 5))
    l = RNG.standard_normal(5)
    rows = np.array([True, False, True, True, False, False])
    y = I.bypass_scale(t, l, rows)
    assert np.allclose(y[rows], t[rows] * l, rtol=1e-14, atol=1e-14)
    assert np.array_equal(y[~rows], t[~rows])


def test_scaled_layer_equals_base_layer_with_folded_weights():
    W, ia3, x = setup(12)
    got = I.forward_seq(CFG, W, ia3, x)
    ref = L.layer_forward_seq(CFG, folded(W, ia3), None, x)
    for name in ("q", "k", "v", "a", "lse", "x2", "gate", "up", "y"):
        assert rel_err(got[name], ref[name]) < 1e-12, name


def test_gradients_match_library_autograd_through_folded_weights():
    """dl of every vector and dX from torch autograd of an independent layer (library ops) whose frozen
    weights carry the vectors as differentiable factors."""
    W, ia3, x = setup(9)
    dY = RNG.standard_normal(x.shape)
    tl = {k: torch.from_numpy(v).requires_grad_() for k, v in ia3.items()}
    tW = {k: torch.from_numpy(v) for k, v in W.items()}
    tWf = dict(tW)
    tWf["wk"], tWf["wv"] = tW["wk"] * tl["k"][:, None], tW["wv"] * tl["v"][:, None]
    tWf["bk"], tWf["bv"] = tW["bk"] * tl["k"], tW["bv"] * tl["v"]
    tWf["wd"] = tW["wd"] * tl["ff"][None, :]
    tx = torch.from_numpy(x).requires_grad_()
    ty = torch_layer(CFG, tWf, {}, tx)
    (ty * torch.from_numpy(dY)).sum().backward()
    dX, g, _, _ = I.backward_seq(CFG, W, ia3, x, dY)
    assert rel_err(dX, tx.grad.numpy()) < 1e-10
    for name in ("k", "v", "ff"):
        assert rel_err(g[name], tl[name].grad.numpy()) < 1e-10, name


def test_gradients_match_central_finite_differences():
    W, ia3, x = setup(7)
    R = RNG.standard_normal(x.shape)
    loss = lambda ia, xx: float(np.sum(I.forward_seq(CFG, W, ia, xx)["y"] * R))
    dX, g, _, _ = I.backward_seq(CFG, W, ia3, x, R)
    h = 1e-6
    for name in ("k", "v", "ff"):
        for j in RNG.choice(ia3[name].size, size=4, replace=False):
            p, m = {k: v.copy() for k, v in ia3.items()}, {k: v.copy() for k, v in ia3.items()}
            p[name][j] += h
            m[name][j] -= h
            fd = (loss(p, x) - loss(m, x)) / (2 * h)
            assert abs(fd - g[name][j]) <= 1e-6 * max(1.0, abs(fd)), (name, j, fd, g[name][j])
    for _ in range(4):
        i, j = RNG.integers(x.shape[0]), RNG.integers(x.shape[1])
        xp, xm = x.copy(), x.copy()
        xp[i, j] += h
        xm[i, j] -= h
        fd = (loss(ia3, xp) - loss(ia3, xm)) / (2 * h)
        assert abs(fd - dX[i, j]) <= 1e-6 * max(1.0, abs(fd))


def token_level(W, ia3, x, dY, fwd, bwd, need_dx=True, ps=4):
    n = x.shape[0]
    pages = np.arange(-(-n // ps))[::-1].copy()
    pool = L.KVPool(len(pages), ps, CFG.kv_dim)
    st = I.Ia3FtState(CFG, n)
    Y = np.zeros_like(x)
    l = 0
    for s in fwd:
        m = build_maps([NS(kind=2, seq_id=0, start_pos=l, n_new=s, adapter=0)], {0: pages}, ps)
        Y[l:l + s] = I.forward_mixed(CFG, W, ia3, m, x[l:l + s], pool, {0: st})
        l += s
    slots = pool.slots(pages, n)
    grads, dX = {}, np.zeros_like(x)
    l = n
    for s in bwd:
        out = I.backward_window(CFG, W, ia3, st, pool.k[slots[:l]], pool.v[slots[:l]], l - s, s, dY[l - s:l], grads, need_dx)
        if need_dx:
            dX[l - s:l] = out
        else:
            assert out is None
        l -= s
    return Y, dX, grads, st


@pytest.mark.parametrize("fwd,bwd", [([11], [11]), ([4, 4, 3], [4, 4, 3]), ([1] * 11, [5, 6]), ([6, 5], [1] * 11),
                                     ([3, 8], [2, 7, 2])])
def test_token_level_equals_whole_sequence(fwd, bwd):
    W, ia3, x = setup(11)
    dY = RNG.standard_normal(x.shape)
    f = I.forward_seq(CFG, W, ia3, x)
    dX, g, dK, dV = I.backward_seq(CFG, W, ia3, x, dY)
    Y, dX_t, g_t, st = token_level(W, ia3, x, dY, fwd, bwd)
    assert rel_err(Y, f["y"]) < 1e-12
    assert rel_err(dX_t, dX) < 1e-11
    for name in ("k", "v", "ff"):
        assert rel_err(g_t[name], g[name]) < 1e-11, name
    assert rel_err(st.dk_accum, dK) < 1e-11 and rel_err(st.dv_accum, dV) < 1e-11
    assert rel_err(st.k0, f["k0"]) < 1e-12 and rel_err(st.v0, f["v0"]) < 1e-12


def test_backward_without_input_grad_still_trains_the_vectors():
    W, ia3, x = setup(8)
    dY = RNG.standard_normal(x.shape)
    _, g, _, _ = I.backward_seq(CFG, W, ia3, x, dY)
    _, _, g_t, _ = token_level(W, ia3, x, dY, [8], [3, 5], need_dx=False)
    for name in ("k", "v", "ff"):
        assert rel_err(g_t[name], g[name]) < 1e-11, name


def test_rows_without_the_adapter_do_not_see_it():
    W, ia3, _ = setup()
    ps = 4
    xs = {0: gen.rng(1, "a", 0).standard_normal((7, CFG.hidden)), 1: gen.rng(1, "a", 1).standard_normal((6, CFG.hidden)),
          2: gen.rng(1, "a", 2).standard_normal((8, CFG.hidden))}
    pages = {0: [4, 1], 1: [0, 5], 2: [3, 2]}
    reqs = [NS(kind=1, seq_id=0, start_pos=0, n_new=7, adapter=-1),       # base-model request
            NS(kind=1, seq_id=1, start_pos=0, n_new=6, adapter=0),        # inference request served with the adapter
            NS(kind=2, seq_id=2, start_pos=0, n_new=8, adapter=0)]        # finetune window
    m = build_maps(reqs, pages, ps)
    pool = L.KVPool(6, ps, CFG.kv_dim)
    st = {2: I.Ia3FtState(CFG, 8)}
    y = I.forward_mixed(CFG, W, ia3, m, np.concatenate([xs[0], xs[1], xs[2]]), pool, st)
    assert rel_err(y[:7], L.layer_forward_seq(CFG, W, None, xs[0])["y"]) < 1e-12
    assert rel_err(y[7:13], I.forward_seq(CFG, W, ia3, xs[1])["y"]) < 1e-12
    assert rel_err(y[13:], I.forward_seq(CFG, W, ia3, xs[2])["y"]) < 1e-12
    other = {k: v * -1.5 for k, v in ia3.items()}
    y2 = I.forward_mixed(CFG, W, other, m, np.concatenate([xs[0], xs[1], xs[2]]), L.KVPool(6, ps, CFG.kv_dim), None)
    assert np.array_equal(y2[:7], y[:7]) and not np.array_equal(y2[7:], y[7:])


def ia3_layer_graph():
    """The decoder layer's operator graph with the three elementwise products of the (IA)^3 network."""
    ops, base, _ = P.decoder_layer_graph(())
    out = []
    for op in ops:
        if op.name == "k_base":
            out += [P.Op("k_base", "matmul", op.inputs, ("k_lin",)), P.Op("k_scale", "mul", ("k_lin", "l_k"), ("k0",), cheap=True)]
        elif op.name == "v_base":
            out += [P.Op("v_base", "matmul", op.inputs, ("v_lin",)), P.Op("v_scale", "mul", ("v_lin", "l_v"), ("v",), cheap=True)]
        elif op.name == "swiglu":
            out += [P.Op("swiglu", "swiglu", op.inputs, ("act0",), cheap=True),
                    P.Op("ff_scale", "mul", ("act0", "l_ff"), ("act",), cheap=True)]
        else:
            out.append(op)
    return out, base, {"l_k", "l_v", "l_ff"}


@pytest.mark.parametrize("need_dx", [True, False])
def test_window_backward_reads_what_graph_pruning_keeps(need_dx):
    ops, base, train = ia3_layer_graph()
    A, R, _ = P.prune(ops, base, train, "y", need_input_grad={"x"} if need_dx else set())
    # (the scaled value rows are one cheap product away from the stored unscaled ones; they sit in the KV
    # cache anyway, which inference needs)
    keep = {"x2", "gate", "up", "q", "k", "k_lin", "v_lin"} | ({"x"} if need_dx else set())
    assert A == keep
    assert {"act0", "v"} <= R and "h2" not in A and "a" not in A
