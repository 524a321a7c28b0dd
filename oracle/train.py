"""The two ends of a finetuning step around the decoder layers (oracle side; test infrastructure).

Alg. 2 computes, for every forward window, a generative loss from the last layer's output rows of
that window, and its backward pass starts from that loss; Sec. 8 (setup) names Adam as the
optimizer of the bypass-network parameters.  The paper fixes neither the loss head nor the
hyper-parameters; the readings here:

  * generative loss = next-token cross-entropy through a final RMSNorm and an LM head,
        h = rmsnorm(x; g),  z = h W_lm^T,  loss_i = logsumexp(z_i) - z_i[y_i],
    summed over the rows whose target y_i >= 0 (a negative target marks "no next token", e.g. the
    last position of a sequence) and scaled by `scale` (1 / tokens of the whole sequence, so that the
    split into windows cannot change the total: the same convention as the MSE head of the layer
    tests);
  * Adam as published (Kingma & Ba, Alg. 1) with bias correction, no weight decay:
        m <- b1 m + (1 - b1) g,  v <- b2 v + (1 - b2) g^2,
        p <- p - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).

Plain numpy in the precision of the arrays handed in (tests use float64).
"""
import numpy as np

from . import ops


def generative_loss(x, g, w_lm, targets, scale, eps):
    """x [n, H]: the window's rows of the last layer's output; g [H]; w_lm [V, H]; targets [n] int
    (a value outside [0, V): the row has no next token and does not count - the paper does not say how such rows
    are marked).  Returns (loss, dx [n, H]) with loss = scale * sum_i loss_i."""
    targets = np.asarray(targets)
    h = ops.rmsnorm(x, g, eps)
    z = h @ w_lm.T
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    se = e.sum(axis=1, keepdims=True)
    lse = (zmax + np.log(se))[:, 0]
    valid = (targets >= 0) & (targets < w_lm.shape[0])
    rows = np.nonzero(valid)[0]
    loss = scale * float(np.sum(lse[rows] - z[rows, targets[rows]]))
    dz = e / se                                  # softmax
    dz[rows, targets[rows]] -= 1.0
    dz[~valid] = 0.0
    dz *= scale
    dh = dz @ w_lm
    return loss, ops.rmsnorm_bwd(x, g, eps, dh)


def adam_step(p, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (step counts from 1).  Returns the new (p, m, v); inputs are not modified."""
    if step < 1:
        raise ValueError("step counts from 1")
    m = beta1 * m + (1.0 - beta1) * grad
    v = beta2 * v + (1.0 - beta2) * grad * grad
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return p - lr * mhat / (np.sqrt(vhat) + eps), m, v


def training_step_whole_seq(cfg, layers, loras, g_final, w_lm, x, targets, scale, opt, step, lr,
                            beta1=0.9, beta2=0.999, eps=1e-8, dtype=np.float64):
    """One sequence-level finetuning step of a stack of decoder layers, written out as its definition:
    forward of the whole sequence through every layer, the generative loss on the top output, backward
    through the layers from the top, then Adam on every bypass matrix.  This is what the token-level
    schedule of Alg. 2 must reproduce whatever its windows (Sec. 6.1).

      layers, loras : per layer the frozen weights and {target: (A, B)}
      x             : [L, H] input rows of the first layer (the frozen embedding's output)
      targets       : [L] next-token ids, negative where a row has none
      opt           : per layer {target: (mA, vA, mB, vB)}; None starts from zeros
    Returns (loss, grads per layer {target: (dA, dB)}, new loras, new opt)."""
    from . import layer as OL
    h = np.asarray(x, dtype=dtype)
    inputs = []
    for W, lo in zip(layers, loras):
        inputs.append(h)
        h = OL.layer_forward_seq(cfg, W, lo, h, dtype)["y"]
    loss, dY = generative_loss(h, np.asarray(g_final, dtype=dtype), np.asarray(w_lm, dtype=dtype), targets, scale, cfg.rms_eps)
    grads = [None] * len(layers)
    for n in range(len(layers) - 1, -1, -1):
        dY, grads[n], _, _ = OL.layer_backward_seq(cfg, layers[n], loras[n], inputs[n], dY, dtype)
    new_loras, new_opt = [], []
    for n, lo in enumerate(loras):
        nl, no = {}, {}
        for t, (A, B) in lo.items():
            A, B = np.asarray(A, dtype=dtype), np.asarray(B, dtype=dtype)
            mA, vA, mB, vB = opt[n][t] if opt is not None else (np.zeros_like(A), np.zeros_like(A), np.zeros_like(B), np.zeros_like(B))
            A1, mA, vA = adam_step(A, grads[n][t][0], mA, vA, step, lr, beta1, beta2, eps)
            B1, mB, vB = adam_step(B, grads[n][t][1], mB, vB, step, lr, beta1, beta2, eps)
            nl[t], no[t] = (A1, B1), (mA, vA, mB, vB)
        new_loras.append(nl)
        new_opt.append(no)
    return loss, grads, new_loras, new_opt
