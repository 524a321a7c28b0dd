"""Static graph pruning (Algorithm 1) on an operator graph (oracle side; test
infrastructure).

Step 1 builds the backward graph by reverse-mode differentiation, deletes every
output that is a gradient of a frozen base weight, shrinks each backward
operator's inputs to what its remaining outputs need, propagates outputs nobody
consumes, and collects A = forward tensors some backward operator still reads.
Step 2 moves a tensor of A to R (rematerialize) when its producer's inputs are
all stored and the producer is cheap.

Readings where the listing is loose:
  * gradients that leave the graph (LoRA weight gradients, and the gradient of
    the graph input when a trainable layer sits below) count as consumed;
  * when an operator's input set shrinks, the producers of the dropped gradient
    tensors are re-examined too (the printed loop re-queues only the operator
    itself, which would stop dead-output propagation after one hop);
  * "inputs stored" in step 2 is tested against A as step 1 left it, weights
    always count as stored, so the outcome does not depend on iteration order;
  * Cost(n) < threshold  :=  n is elementwise, a norm, or a rank-r matmul;
  * attention is one operator whose backward reads Q, K, V and recomputes the
    softmax probabilities internally;
  * other bypass networks (Sec. 4.1 names (IA)^3 and bottleneck adapters beside LoRA) need two more
    operator kinds: `mul`, the elementwise product with a learned vector, and `relu`, whose backward
    reads only the sign of its output: 'm:<t>' denotes that sign bitmask of tensor t (the compressed
    form Sec. 5.2 mentions for ReLU), which a tensor needed by nobody else is stored as.
The worked example of the paper's pruning figure (MLP with LoRA) is not available
in the text: that example is parity unpinned; the tests pin this code against an
independent demand-driven reachability search instead.
"""
from collections import deque
from dataclasses import dataclass, field
from typing import Dict, List, Set, Tuple


@dataclass
class Op:
    name: str
    kind: str                 # matmul | add | rmsnorm | rope | attention | swiglu | mul | relu | source
    inputs: Tuple[str, ...]
    outputs: Tuple[str, ...]
    cheap: bool = False


def grad_rules(op: Op) -> Dict[str, Set[str]]:
    """Reverse-mode rule of one forward operator: for each input, the tensors its
    gradient is computed from ('d:<t>' denotes the gradient of tensor t)."""
    o = op.outputs[0] if op.outputs else None
    i = op.inputs
    if op.kind == "source":
        return {}
    if op.kind == "matmul":           # y = x @ w
        x, w = i
        return {x: {"d:" + o, w}, w: {"d:" + o, x}}
    if op.kind == "add":
        return {t: {"d:" + o} for t in i}
    if op.kind == "rmsnorm":          # h = rmsnorm(x; g)
        x, g = i
        return {x: {"d:" + o, x, g}, g: {"d:" + o, x}}
    if op.kind == "rope":
        return {i[0]: {"d:" + o}}
    if op.kind == "attention":        # a = attn(q, k, v)
        return {t: {"d:" + o, *i} for t in i}
    if op.kind == "swiglu":           # act = silu(gate) * up
        g, u = i
        return {g: {"d:" + o, g, u}, u: {"d:" + o, g}}
    if op.kind == "mul":              # y = a * b, elementwise
        a, b = i
        return {a: {"d:" + o, b}, b: {"d:" + o, a}}
    if op.kind == "relu":             # y = max(x, 0): the gradient passes where y > 0
        return {i[0]: {"d:" + o, "m:" + o}}
    raise ValueError(op.kind)


def prune(ops: List[Op], base_weights: Set[str], trainable: Set[str], graph_output: str,
          need_input_grad: Set[str] = frozenset()):
    """Returns (A, R, A_step1).  trainable: LoRA weights; need_input_grad: source
    tensors whose gradient is handed to a layer below."""
    A, R, A1, _ = prune_with_masks(ops, base_weights, trainable, graph_output, need_input_grad)
    return A, R, A1


def prune_with_masks(ops: List[Op], base_weights: Set[str], trainable: Set[str], graph_output: str,
                     need_input_grad: Set[str] = frozenset()):
    """Returns (A, R, A_step1, M): M = forward tensors of which only the sign bitmask is read."""
    fwd_out = {t for op in ops for t in op.outputs}
    producer = {t: op for op in ops for t in op.outputs}
    weights = set(base_weights) | set(trainable)
    # ---- ReverseAutoDiff: one backward operator per forward operator ----------
    rules = {op.name: grad_rules(op) for op in ops}
    b_out = {op.name: {"d:" + t for t in rules[op.name]} for op in ops}
    sinks = {"d:" + t for t in trainable} | {"d:" + t for t in need_input_grad}

    def update_input(name):
        need = set()
        for t in b_out[name]:
            need |= rules[name][t[2:]]
        return need

    b_in = {op.name: update_input(op.name) for op in ops}
    grad_producers = {}
    for op in ops:
        for t in b_out[op.name]:
            grad_producers.setdefault(t, set()).add(op.name)
    Q = deque()

    def shrink(name):
        old = b_in[name]
        b_in[name] = update_input(name)
        Q.append(name)
        for t in old - b_in[name]:
            for p in grad_producers.get(t, ()):
                Q.append(p)

    # ---- drop gradients of frozen base weights --------------------------------
    for op in ops:
        for t in list(b_out[op.name]):
            if t[2:] in base_weights:
                b_out[op.name].discard(t)
                shrink(op.name)
    # ---- propagate outputs nobody reads ----------------------------------------
    while Q:
        name = Q.popleft()
        for t in list(b_out[name]):
            consumed = t in sinks or any(t in b_in[u] for u in b_in)
            if not consumed:
                b_out[name].discard(t)
                shrink(name)
    A1 = {t for t in fwd_out if any(t in b_in[u] for u in b_in)}
    M = {t for t in fwd_out if t not in A1 and any("m:" + t in b_in[u] for u in b_in)}
    # ---- step 2: rematerialization ---------------------------------------------
    A, R = set(A1), set()
    for t in sorted(A1):
        n = producer[t]
        if n.kind != "source" and n.cheap and all((x in A1) or (x in weights) for x in n.inputs):
            A.discard(t)
            R.add(t)
    return A, R, A1, M


def decoder_layer_graph(lora_targets, rank_cheap=True):
    """Operator graph of the LoRA-augmented decoder layer used in this repository
    (one LLaMA/Qwen-style layer; each LoRA bypass is two matmuls and an add)."""
    ops = [Op("input", "source", (), ("x",))]
    base, train = set(), set()

    def linear(tag, xin, wname, out):
        base.add(wname)
        if tag in lora_targets:
            A, B = f"A_{tag}", f"B_{tag}"
            train.update((A, B))
            ops.append(Op(f"{tag}_base", "matmul", (xin, wname), (f"{out}_base",)))
            ops.append(Op(f"{tag}_shrink", "matmul", (xin, A), (f"u_{tag}",), cheap=rank_cheap))
            ops.append(Op(f"{tag}_expand", "matmul", (f"u_{tag}", B), (f"l_{tag}",), cheap=rank_cheap))
            ops.append(Op(f"{tag}_add", "add", (f"{out}_base", f"l_{tag}"), (out,), cheap=True))
        else:
            ops.append(Op(f"{tag}_base", "matmul", (xin, wname), (out,)))

    base.update(("g1", "g2"))
    ops.append(Op("norm1", "rmsnorm", ("x", "g1"), ("h1",), cheap=True))
    linear("q", "h1", "Wq", "q0")
    linear("k", "h1", "Wk", "k0")
    linear("v", "h1", "Wv", "v")
    ops.append(Op("rope_q", "rope", ("q0",), ("q",), cheap=True))
    ops.append(Op("rope_k", "rope", ("k0",), ("k",), cheap=True))
    ops.append(Op("attn", "attention", ("q", "k", "v"), ("a",)))
    linear("o", "a", "Wo", "o_out")
    ops.append(Op("res1", "add", ("x", "o_out"), ("x2",), cheap=True))
    ops.append(Op("norm2", "rmsnorm", ("x2", "g2"), ("h2",), cheap=True))
    linear("gate", "h2", "Wg", "gate")
    linear("up", "h2", "Wu", "up")
    ops.append(Op("swiglu", "swiglu", ("gate", "up"), ("act",), cheap=True))
    linear("down", "act", "Wd", "d_out")
    ops.append(Op("res2", "add", ("x2", "d_out"), ("y",), cheap=True))
    return ops, base, train


def prune_decoder_layer(lora_targets, need_dx=True):
    ops, base, train = decoder_layer_graph(tuple(lora_targets))
    return prune(ops, base, train, "y", need_input_grad={"x"} if need_dx else set())
