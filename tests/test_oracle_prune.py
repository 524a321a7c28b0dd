"""Pins for oracle/prune.py (Algorithm 1): the hand-derived activation set of the
decoder layer, and an independent demand-driven search for what the kept gradients
depend on.  The paper's own worked example (its pruning figure) is not in the text:
that example stays unpinned."""
import pytest

from oracle import prune as P


@pytest.mark.parametrize("targets,expect_A", [
    (("down",), {"x2", "gate", "up", "q", "k", "v", "x"}),
    (("q", "v", "down"), {"x", "x2", "gate", "up", "q", "k", "v"}),
    (("q", "k", "v", "o", "down"), {"x", "x2", "gate", "up", "q", "k", "v", "a"}),
    (("q", "k", "v", "o", "gate", "up", "down"), {"x", "x2", "gate", "up", "q", "k", "v", "a"}),
])
def test_decoder_layer_sets(targets, expect_A):
    A, R, A1 = P.prune_decoder_layer(targets, need_dx=True)
    assert A == expect_A
    # rematerialized: the norm outputs and SwiGLU product when a LoRA input needs them,
    # and every low-rank intermediate
    for t in targets:
        assert f"u_{t}" in R
    if "down" in targets:
        assert "act" in R
    if any(t in targets for t in ("q", "k", "v")):
        assert "h1" in R
    if any(t in targets for t in ("gate", "up")):
        assert "h2" in R
    assert A.isdisjoint(R) and (A | R) == A1


def test_bottom_layer_drops_input_side():
    # only the down projection is trainable and nothing below needs dX: the whole
    # attention side and the SwiGLU backward are dead; dA needs act itself (its
    # producer's inputs gate, up are no longer stored, so it cannot be rematerialized)
    A, R, _ = P.prune_decoder_layer(("down",), need_dx=False)
    assert A == {"act"} and R == {"u_down"}
    # with LoRA on q the attention inputs are needed again, and h1 itself (the norm's
    # backward is dead, so x is not stored and h1 cannot be recomputed from it)
    A, R, _ = P.prune_decoder_layer(("q", "down"), need_dx=False)
    assert A == {"h1", "q", "k", "v", "x2", "gate", "up"} and R == {"act", "u_down", "u_q"}


def demand_closure(ops, base, train, need_input_grad):
    """Independent check: starting from the gradients that must be produced, follow
    'to compute the gradient of t I need ...' recursively (top-down), and collect
    the forward activations touched."""
    consumers = {}
    for op in ops:
        for t in op.inputs:
            consumers.setdefault(t, []).append(op)
    fwd_out = {t for op in ops for t in op.outputs}
    need_fwd, need_mask, seen = set(), set(), set()

    def need_grad(t):
        if t in seen:
            return
        seen.add(t)
        for op in consumers.get(t, []):          # dL/dt sums over every consumer of t
            for dep in P.grad_rules(op)[t]:
                if dep.startswith("d:"):
                    need_grad(dep[2:])
                elif dep.startswith("m:"):
                    need_mask.add(dep[2:])
                elif dep in fwd_out:
                    need_fwd.add(dep)

    for t in list(train) + list(need_input_grad):
        need_grad(t)
    demand_closure.masks = need_mask - need_fwd
    return need_fwd


@pytest.mark.parametrize("targets", [("down",), ("q", "v", "down"), ("o",), ("gate", "up"),
                                     ("q", "k", "v", "o", "gate", "up", "down")])
@pytest.mark.parametrize("need_dx", [True, False])
def test_step1_equals_demand_driven_search(targets, need_dx):
    ops, base, train = P.decoder_layer_graph(targets)
    _, _, A1 = P.prune(ops, base, train, "y", need_input_grad={"x"} if need_dx else set())
    assert A1 == demand_closure(ops, base, train, {"x"} if need_dx else set())


def test_full_finetuning_keeps_everything_a_weight_gradient_needs():
    # with no frozen weight, nothing is pruned: every matmul input stays
    ops, base, train = P.decoder_layer_graph(())
    A, R, A1 = P.prune(ops, set(), base, "y", need_input_grad={"x"})
    assert {"h1", "a", "h2", "act", "x", "x2", "gate", "up", "q", "k", "v"} <= A1


def test_mlp_with_lora_toy_graph():
    """y = relu-free toy: h = x W1 (frozen); z = h W2 (frozen) + (h A) B.  The gradient
    of A needs h; dh needs only weights; x is needed by nobody (dW1 is pruned)."""
    ops = [P.Op("in", "source", (), ("x",)),
           P.Op("l1", "matmul", ("x", "W1"), ("h",)),
           P.Op("l2", "matmul", ("h", "W2"), ("z0",)),
           P.Op("sh", "matmul", ("h", "A"), ("u",), cheap=True),
           P.Op("ex", "matmul", ("u", "B"), ("zl",), cheap=True),
           P.Op("add", "add", ("z0", "zl"), ("z",), cheap=True)]
    A, R, A1 = P.prune(ops, {"W1", "W2"}, {"A", "B"}, "z")
    assert A1 == {"h", "u"} and A == {"h"} and R == {"u"}


def ia3_graph():
    """(IA)^3 on the keys of a frozen projection, k = (h Wk) * l_k with l_k learned, followed by a frozen
    consumer; and a frozen ReLU MLP above it."""
    return [P.Op("in", "source", (), ("h",)),
            P.Op("k_base", "matmul", ("h", "Wk"), ("k0",)),
            P.Op("k_scale", "mul", ("k0", "l_k"), ("k",), cheap=True),
            P.Op("fc1", "matmul", ("k", "W1"), ("z1",)),
            P.Op("act", "relu", ("z1",), ("r1",), cheap=True),
            P.Op("fc2", "matmul", ("r1", "W2"), ("y",))]


def test_ia3_and_relu_bitmask():
    """The gradient of l_k is sum over rows of dk * k0: k0 is kept in full.  The frozen ReLU MLP above
    only passes the gradient through: of r1 only the sign bitmask is kept, z1 and k not at all."""
    A, R, A1, M = P.prune_with_masks(ia3_graph(), {"Wk", "W1", "W2"}, {"l_k"}, "y")
    assert A1 == {"k0"} and A == {"k0"} and R == set() and M == {"r1"}
    # with a trainable layer below, h is still not needed (dh = dk0 Wk^T reads only the weight)
    A, R, A1, M = P.prune_with_masks(ia3_graph(), {"Wk", "W1", "W2"}, {"l_k"}, "y", need_input_grad={"h"})
    assert A1 == {"k0"} and M == {"r1"}


def test_bottleneck_adapter_keeps_its_relu_output_in_full():
    """Adapter y = x1 + relu(x1 Wd) Wu on top of a frozen projection x1 = x W: dWu needs relu's output in
    full (so no bitmask), dWd needs x1; x itself is needed by nobody."""
    ops = [P.Op("in", "source", (), ("x",)),
           P.Op("base", "matmul", ("x", "W"), ("x1",)),
           P.Op("down", "matmul", ("x1", "Wd"), ("z",), cheap=True),
           P.Op("act", "relu", ("z",), ("r",), cheap=True),
           P.Op("up", "matmul", ("r", "Wu"), ("a",), cheap=True),
           P.Op("add", "add", ("x1", "a"), ("y",), cheap=True)]
    A, R, A1, M = P.prune_with_masks(ops, {"W"}, {"Wd", "Wu"}, "y")
    assert A1 == {"x1", "r"} and M == set()
    # r = relu(z) is cheap but its input z is not stored: it stays stored itself
    assert A == {"x1", "r"} and R == set()


@pytest.mark.parametrize("need_dx", [True, False])
def test_step1_equals_demand_driven_search_with_masks(need_dx):
    ops = ia3_graph()
    nig = {"h"} if need_dx else set()
    _, _, A1, M = P.prune_with_masks(ops, {"Wk", "W1", "W2"}, {"l_k"}, "y", need_input_grad=nig)
    assert A1 == demand_closure(ops, {"Wk", "W1", "W2"}, {"l_k"}, nig)
    assert M == demand_closure.masks
