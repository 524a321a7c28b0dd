"""A bottleneck adapter as a bypass network (oracle side; test infrastructure).

Sec. 4.1 represents every PEFT method as bypass networks: each takes ONE backbone tensor X and its
output is added to one backbone tensor, Y = f_B(X) + f_A(X).  The adapter modules of the PEFT
literature the paper lists (Sec. 2) are a down-projection to a small width b, a ReLU, and an
up-projection back:  f_A(X) = relu(X W_down^T) W_up^T.  Reading taken here (the paper names adapters
without fixing where they attach): the adapter sits on a layer's output rows, X = the layer output,
f_B = identity, so Y = X + relu(X W_down^T) W_up^T on the rows of requests that carry the adapter
and Y = X elsewhere; no biases.  W_down [b, H], W_up [H, b] are the only trainable parameters.

The network is row-local, so Algorithm 2's token windows need no cache for it: a window's backward
reads the window's own stored input rows X (what graph pruning keeps; the ReLU output is recomputed
from them through two cheap operators) and the incoming gradient rows.
"""
import numpy as np


def forward(x, w_down, w_up, rows=None):
    """x [n, H]; rows: boolean mask of the rows that carry the adapter (None: all)."""
    x = np.asarray(x)
    y = x.copy()
    sel = np.ones(x.shape[0], dtype=bool) if rows is None else np.asarray(rows, dtype=bool)
    z = x[sel] @ w_down.T
    r = np.maximum(z, 0.0)
    y[sel] = x[sel] + r @ w_up.T
    return y


def backward(x, w_down, w_up, dy):
    """Every row of x carries the adapter.  Returns (dx, dw_down, dw_up) for Y = X + relu(X W_down^T) W_up^T."""
    z = x @ w_down.T
    r = np.maximum(z, 0.0)
    dr = dy @ w_up
    dz = dr * (z > 0.0)
    return dy + dz @ w_down, dz.T @ x, dy.T @ r
