"""Pins of the loss-head and optimizer oracle: finite differences, closed forms and invariants."""
import numpy as np
import pytest

from oracle import train as T
from workload import gen


def setup(seed, n=7, H=24, V=53):
    g = gen.rng(seed, "train", "head", n, H, V)
    x = g.standard_normal((n, H))
    gain = 1.0 + 0.1 * g.standard_normal(H)
    w = 0.3 * g.standard_normal((V, H))
    y = g.integers(0, V, n)
    return x, gain, w, y


def test_loss_of_a_zero_head_is_log_vocab():
    x, gain, w, y = setup(0)
    loss, dx = T.generative_loss(x, gain, np.zeros_like(w), y, 1.0 / len(y), 1e-5)
    assert loss == pytest.approx(np.log(w.shape[0]), rel=1e-12)
    assert np.abs(dx).max() == 0.0                     # the logits do not depend on x


def test_loss_gradient_matches_central_differences():
    x, gain, w, y = setup(1)
    y[2] = -1                                          # one ignored row
    scale = 1.0 / 11.0
    loss, dx = T.generative_loss(x, gain, w, y, scale, 1e-5)
    num = np.zeros_like(x)
    h = 1e-6
    for i in range(x.shape[0]):
        for j in range(x.shape[1]):
            xp, xm = x.copy(), x.copy()
            xp[i, j] += h
            xm[i, j] -= h
            num[i, j] = (T.generative_loss(xp, gain, w, y, scale, 1e-5)[0] - T.generative_loss(xm, gain, w, y, scale, 1e-5)[0]) / (2 * h)
    assert np.abs(dx - num).max() <= 1e-8 * max(1.0, np.abs(num).max())
    assert np.abs(dx[2]).max() == 0.0                  # the ignored row gets no gradient


def test_loss_is_the_textbook_cross_entropy_and_additive_over_windows():
    x, gain, w, y = setup(2, n=10)
    from oracle import ops
    z = ops.rmsnorm(x, gain, 1e-5) @ w.T
    p = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    want = -np.log(p[np.arange(10), y]).sum() / 10
    whole, dx = T.generative_loss(x, gain, w, y, 0.1, 1e-5)
    assert whole == pytest.approx(want, rel=1e-12)
    a, dxa = T.generative_loss(x[:4], gain, w, y[:4], 0.1, 1e-5)
    b, dxb = T.generative_loss(x[4:], gain, w, y[4:], 0.1, 1e-5)
    assert a + b == pytest.approx(whole, rel=1e-12)    # windows of a sequence add up (Alg. 2, forward loop)
    assert np.allclose(np.vstack([dxa, dxb]), dx, rtol=1e-12, atol=0)


def test_rows_with_a_target_outside_the_vocabulary_do_not_count():
    x, gain, w, y = setup(4, n=9)
    V = w.shape[0]
    keep = np.array([0, 2, 3, 5, 8])
    y2 = y.copy()
    y2[1], y2[4], y2[6], y2[7] = -1, V, V + 1000, -7
    got, dx = T.generative_loss(x, gain, w, y2, 0.2, 1e-5)
    want, dxk = T.generative_loss(x[keep], gain, w, y[keep], 0.2, 1e-5)      # rows are independent: drop them instead
    assert got == pytest.approx(want, rel=1e-12)
    assert np.allclose(dx[keep], dxk, rtol=1e-12, atol=0)
    assert np.all(dx[[1, 4, 6, 7]] == 0.0)


def test_loss_is_stable_for_large_logits():
    x, gain, w, y = setup(3)
    loss, dx = T.generative_loss(x, gain, 400.0 * w, y, 1.0, 1e-5)
    assert np.isfinite(loss) and np.isfinite(dx).all()


def test_adam_first_step_moves_by_lr_against_the_sign():
    g = gen.rng(4, "train", "adam")
    p, grad = g.standard_normal(50), g.standard_normal(50)
    p1, m1, v1 = T.adam_step(p, grad, np.zeros(50), np.zeros(50), 1, lr=1e-2, eps=0.0)
    assert np.allclose(p1, p - 1e-2 * np.sign(grad), rtol=1e-12)
    assert np.allclose(m1, 0.1 * grad) and np.allclose(v1, 0.001 * grad * grad)


def test_adam_with_a_constant_gradient_has_unit_normalised_steps():
    """m_hat = g and v_hat = g^2 at every step when the gradient never changes: each step is
    lr * g / (|g| + eps)."""
    grad = np.array([0.5, -2.0, 1e-3])
    p, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    for t in range(1, 8):
        p, m, v = T.adam_step(p, grad, m, v, t, lr=0.1, eps=1e-8)
        assert np.allclose(p, -0.1 * t * grad / (np.abs(grad) + 1e-8), rtol=1e-10)


def test_adam_minimises_a_quadratic_and_rejects_step_zero():
    target = np.array([3.0, -1.0])
    p, m, v = np.zeros(2), np.zeros(2), np.zeros(2)
    for t in range(1, 3001):
        p, m, v = T.adam_step(p, 2 * (p - target), m, v, t, lr=0.01)
    assert np.abs(p - target).max() < 1e-3
    with pytest.raises(ValueError):
        T.adam_step(p, p, m, v, 0, lr=0.1)


def test_whole_sequence_step_gradients_match_central_differences_through_two_layers():
    """Pins the composition (layer order, the loss head on top, gradients routed to the right layer and
    matrix): d loss / d(entry of A or B) by central differences of the loss alone."""
    from workload import CONFIGS
    cfg = CONFIGS["c1_tiny_f32"].with_(hidden=32, n_q_heads=2, n_kv_heads=1, head_dim=16, ffn=40, lora_rank=2,
                                       lora_targets=("q", "v", "o", "down"))
    L, V = 9, 31
    layers = [gen.layer_weights(cfg, 5, n) for n in range(2)]
    loras = [gen.lora_weights(cfg, 5, n, b_std=0.05) for n in range(2)]
    layers = [{k: v.astype(np.float64) for k, v in W.items()} for W in layers]
    loras = [{t: (A.astype(np.float64), B.astype(np.float64)) for t, (A, B) in lo.items()} for lo in loras]
    g = gen.rng(5, "train", "step")
    x = g.standard_normal((L, cfg.hidden))
    gain = 1.0 + 0.1 * g.standard_normal(cfg.hidden)
    w = 0.3 * g.standard_normal((V, cfg.hidden))
    y = g.integers(0, V, L)
    y[-1] = -1
    loss, grads, new_loras, new_opt = T.training_step_whole_seq(cfg, layers, loras, gain, w, x, y, 1.0 / L, None, 1, 1e-2)

    def loss_with(n, t, which, idx, delta):
        lo2 = [{k: (A.copy(), B.copy()) for k, (A, B) in lo.items()} for lo in loras]
        lo2[n][t][which][idx] += delta
        return T.training_step_whole_seq(cfg, layers, lo2, gain, w, x, y, 1.0 / L, None, 1, 1e-2)[0]

    h = 1e-5
    checked = 0
    for n in range(2):
        for t in cfg.lora_targets:
            for which in (0, 1):
                shape = loras[n][t][which].shape
                for _ in range(2):
                    idx = (int(g.integers(0, shape[0])), int(g.integers(0, shape[1])))
                    num = (loss_with(n, t, which, idx, h) - loss_with(n, t, which, idx, -h)) / (2 * h)
                    got = grads[n][t][which][idx]
                    assert abs(got - num) <= 1e-6 * max(1e-3, abs(num)) + 1e-10, (n, t, which, idx, got, num)
                    checked += 1
    assert checked == 32
    # first Adam step from zero state: m_hat = g, v_hat = g^2, so every entry moves by lr g / (|g| + eps)
    for n in range(2):
        for t in cfg.lora_targets:
            for which in (0, 1):
                gr = grads[n][t][which]
                moved = new_loras[n][t][which] - loras[n][t][which]
                assert np.allclose(moved, -1e-2 * gr / (np.abs(gr) + 1e-8), rtol=1e-9, atol=1e-15)
