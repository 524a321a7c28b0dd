"""Pins for oracle/adapter.py (the bottleneck adapter as a bypass network, Sec. 4.1): a zero up-projection
is the identity; library autograd; central finite differences; row locality (windows = whole sequence,
rows without the adapter untouched); the pruner keeps the adapter's input and nothing it cannot derive."""
import numpy as np
import torch

from oracle import adapter as A
from oracle import prune as P

RNG = np.random.default_rng(31)


def setup(n=9, H=24, b=6):
    return RNG.standard_normal((n, H)), RNG.standard_normal((b, H)) * 0.4, RNG.standard_normal((H, b)) * 0.4


def test_zero_up_projection_is_the_identity_and_stops_the_down_gradient():
    x, wd, wu = setup()
    y = A.forward(x, wd, np.zeros_like(wu))
    assert np.array_equal(y, x)
    dx, dwd, dwu = A.backward(x, wd, np.zeros_like(wu), RNG.standard_normal(x.shape))
    assert np.all(dwd == 0.0) and np.any(dwu != 0.0)


def test_matches_library_autograd():
    x, wd, wu = setup()
    dy = RNG.standard_normal(x.shape)
    tx, twd, twu = (torch.from_numpy(a).requires_grad_() for a in (x, wd, wu))
    ty = tx + torch.nn.functional.linear(torch.relu(torch.nn.functional.linear(tx, twd)), twu)
    (ty * torch.from_numpy(dy)).sum().backward()
    assert np.allclose(A.forward(x, wd, wu), ty.detach().numpy(), rtol=1e-13, atol=1e-13)
    dx, dwd, dwu = A.backward(x, wd, wu, dy)
    for got, ref in ((dx, tx.grad), (dwd, twd.grad), (dwu, twu.grad)):
        assert np.allclose(got, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_gradients_match_central_finite_differences():
    x, wd, wu = setup(5, 10, 4)
    R = RNG.standard_normal(x.shape)
    loss = lambda xx, a, b: float(np.sum(A.forward(xx, a, b) * R))
    dx, dwd, dwu = A.backward(x, wd, wu, R)
    h = 1e-6
    for arr, grad, which in ((x, dx, 0), (wd, dwd, 1), (wu, dwu, 2)):
        for _ in range(5):
            i, j = RNG.integers(arr.shape[0]), RNG.integers(arr.shape[1])
            args = [x.copy(), wd.copy(), wu.copy()]
            args[which][i, j] += h
            up = loss(*args)
            args[which][i, j] -= 2 * h
            fd = (up - loss(*args)) / (2 * h)
            assert abs(fd - grad[i, j]) <= 1e-6 * max(1.0, abs(fd)), (which, i, j)


def test_row_local_windows_and_rows_without_the_adapter():
    x, wd, wu = setup(11)
    dy = RNG.standard_normal(x.shape)
    dx, dwd, dwu = A.backward(x, wd, wu, dy)
    gd, gu, dxs = np.zeros_like(wd), np.zeros_like(wu), np.zeros_like(x)
    l = 11
    for s in (3, 1, 7):                               # windows from the sequence end (Alg. 2)
        a, b, c = A.backward(x[l - s:l], wd, wu, dy[l - s:l])
        dxs[l - s:l], gd, gu = a, gd + b, gu + c
        l -= s
    assert np.allclose(dxs, dx, rtol=1e-13, atol=1e-13)
    assert np.allclose(gd, dwd, rtol=1e-12, atol=1e-12) and np.allclose(gu, dwu, rtol=1e-12, atol=1e-12)
    rows = np.arange(11) % 3 == 0
    y = A.forward(x, wd, wu, rows)
    assert np.array_equal(y[~rows], x[~rows])
    assert np.allclose(y[rows], A.forward(x[rows], wd, wu), rtol=1e-14, atol=1e-14)


def test_graph_pruning_keeps_the_adapter_input():
    ops = [P.Op("in", "source", (), ("x",)),
           P.Op("down", "matmul", ("x", "Wd"), ("z",), cheap=True),
           P.Op("act", "relu", ("z",), ("r",), cheap=True),
           P.Op("up", "matmul", ("r", "Wu"), ("a",), cheap=True),
           P.Op("add", "add", ("x", "a"), ("y",), cheap=True)]
    A_, R_, _, M_ = P.prune_with_masks(ops, set(), {"Wd", "Wu"}, "y", need_input_grad={"x"})
    # x is stored (the down-projection's weight gradient reads it); z is one cheap operator away from it, and
    # with z back the ReLU output is too: the implementation stores x alone and recomputes both
    assert "x" in A_ and "z" not in A_ and not M_
    assert A_ <= {"x", "r"}
