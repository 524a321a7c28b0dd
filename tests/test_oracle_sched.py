"""Pins of the scheduler oracle (Sec. 6.2, Hybrid Token Scheduler) against what the paper and the
mathematics fix: the interpolant reproduces its table and any bilinear function, the window rule is
the closed form for a linear latency model and a brute-force argmax otherwise, and the inference
stage serves a hand-worked example and keeps its invariants on random request streams."""
import numpy as np
import pytest

from oracle import sched as S
from workload import gen


def grids():
    return [0, 64, 256, 512, 1024], [0, 32, 128, 256, 512]


def table(fn, cg, sg):
    return [[fn(c, s) for s in sg] for c in cg]


def test_estimate_reproduces_the_table():
    cg, sg = grids()
    g = gen.rng(1, "sched", "table")
    ms = (g.random((len(cg), len(sg))) * 50 + 1).tolist()
    for i, c in enumerate(cg):
        for j, s in enumerate(sg):
            assert S.latency_estimate(cg, sg, ms, c, s) == pytest.approx(ms[i][j], rel=1e-13)


@pytest.mark.parametrize("a,b,d,e", [(3.0, 0.02, 0.03, 0.0), (1.5, 0.01, 0.04, 2e-5), (0.0, 0.0, 0.1, 0.0)])
def test_estimate_is_exact_for_bilinear_functions_inside_and_outside_the_grid(a, b, d, e):
    fn = lambda c, s: a + b * c + d * s + e * c * s
    cg, sg = grids()
    ms = table(fn, cg, sg)
    g = gen.rng(2, "sched", "bilinear", a, b, d, e)
    for c, s in zip(g.integers(0, 2000, 200), g.integers(0, 900, 200)):   # beyond both grids too
        assert S.latency_estimate(cg, sg, ms, int(c), int(s)) == pytest.approx(fn(c, s), rel=1e-11, abs=1e-11)


def test_estimate_uses_the_segment_that_contains_the_point():
    # a kink at c = 256: left slope 1, right slope 3 (s plays no role)
    cg, sg = [0, 256, 512], [0, 100]
    ms = [[0.0, 0.0], [256.0, 256.0], [1024.0, 1024.0]]
    assert S.latency_estimate(cg, sg, ms, 128, 50) == pytest.approx(128.0)
    assert S.latency_estimate(cg, sg, ms, 384, 50) == pytest.approx(256.0 + 3 * 128.0)
    assert S.latency_estimate(cg, sg, ms, 640, 50) == pytest.approx(1024.0 + 3 * 128.0)   # last segment extended


@pytest.mark.parametrize("quantum", [1, 16, 64])
def test_window_is_the_closed_form_for_a_linear_model(quantum):
    """f = a + b c + d s with d > 0:  the largest candidate s with s <= (SLO - a - b c) / d."""
    a, b, d = 4.0, 0.03, 0.05
    cg, sg = grids()
    ms = table(lambda c, s: a + b * c + d * s, cg, sg)
    g = gen.rng(3, "sched", "linear", quantum)
    for _ in range(300):
        c = int(g.integers(0, 1500))
        slo = float(g.uniform(0.0, 120.0))
        s_avail = int(g.integers(0, 700))
        bound = (slo - a - b * c) / d
        cands = sorted(set(list(range(0, s_avail + 1, quantum)) + [s_avail]))
        want = max([s for s in cands if s <= bound + 1e-9], default=0)
        got = S.pick_window(cg, sg, ms, c, slo, s_avail, quantum)
        # the closed form and the estimate may disagree only within rounding of the bound itself
        if abs(bound - round(bound)) > 1e-6:
            assert got == want, (c, slo, s_avail, bound)
        assert got in cands
        assert got == 0 or S.latency_estimate(cg, sg, ms, c, got) <= slo


def test_window_edge_cases():
    cg, sg = grids()
    ms = table(lambda c, s: 10.0 + 0.1 * s, cg, sg)
    assert S.pick_window(cg, sg, ms, 100, 9.99, 512, 16) == 0            # even s = 0 misses the SLO
    assert S.pick_window(cg, sg, ms, 100, 10.0, 512, 16) == 0            # only s = 0 meets it
    assert S.pick_window(cg, sg, ms, 100, 1e9, 500, 16) == 500           # s_avail itself is a candidate
    assert S.pick_window(cg, sg, ms, 100, 1e9, 0, 16) == 0
    assert S.pick_window(cg, sg, ms, 100, 10.0 + 0.1 * 48, 512, 16) == 48
    with pytest.raises(ValueError):
        S.pick_window(cg, sg, ms, 100, 20.0, 64, 0)


def test_window_is_an_argmax_not_a_first_failure_search():
    """A profiled table need not be monotone: the rule is the largest s that meets the SLO."""
    cg, sg = [0, 1000], [0, 100, 200, 300]
    ms = [[1.0, 9.0, 2.0, 9.0], [1.0, 9.0, 2.0, 9.0]]
    assert S.pick_window(cg, sg, ms, 500, 5.0, 300, 100) == 200


def test_inference_stage_hand_worked_example():
    """Three requests (prompt, generate): A (5, 2), B (3, 1), C (4, 2); at most 2 running, 4 tokens per
    iteration, chunks of at most 3.  Worked by hand from the rules of Sec. 6.2."""
    P, D = S.KIND_PREFILL, S.KIND_DECODE
    prompt, gen_len = [5, 3, 4], [2, 1, 2]
    prefilled, generated, state = [0, 0, 0], [0, 0, 0], [S.WAITING] * 3
    expect = [
        [(0, P, 0, 3), (1, P, 0, 1)],          # A and B admitted; B gets what is left of the budget
        [(0, P, 3, 2), (1, P, 1, 2)],          # both prompts complete
        [(0, D, 5, 1), (1, D, 3, 1)],          # both generate; C still waits (2 running)
        [(0, D, 6, 1), (2, P, 0, 3)],          # B finished -> C admitted; decode entries first
        [(2, P, 3, 1)],                        # A finished
        [(2, D, 4, 1)],
        [(2, D, 5, 1)],
    ]
    for it, want in enumerate(expect):
        got = S.schedule_inference(prompt, prefilled, gen_len, generated, state, max_batch=2, token_budget=4, chunk=3)
        assert got == want, it
        S.apply_iteration(got, prompt, prefilled, gen_len, generated, state)
    assert state == [S.FINISHED] * 3
    assert S.schedule_inference(prompt, prefilled, gen_len, generated, state, 2, 4, 3) == []


@pytest.mark.parametrize("seed,max_batch,budget,chunk", [(0, 4, 64, 16), (1, 8, 32, 32), (2, 1, 7, 3), (3, 16, 256, 64)])
def test_inference_stage_invariants_on_random_streams(seed, max_batch, budget, chunk):
    g = gen.rng(seed, "sched", "stream")
    n = 40
    prompt = [int(x) for x in g.integers(1, 200, n)]
    gen_len = [int(x) for x in g.integers(0, 30, n)]
    prefilled, generated, state = [0] * n, [0] * n, [S.WAITING] * n
    got_prefill, got_decode = [0] * n, [0] * n
    first_seen = {}
    for it in range(100000):
        entries = S.schedule_inference(prompt, prefilled, gen_len, generated, state, max_batch, budget, chunk)
        if not entries and all(st != S.RUNNING for st in state):
            break
        assert sum(e[3] for e in entries) <= budget
        assert sum(1 for st in state if st == S.RUNNING) <= max_batch
        kinds = [e[1] for e in entries]
        assert kinds == sorted(kinds)                              # decode entries first
        for (r, kind, start, n_new) in entries:
            first_seen.setdefault(r, it)
            assert n_new >= 1 and state[r] == S.RUNNING
            if kind == S.KIND_PREFILL:
                assert start == got_prefill[r] and n_new <= chunk
                got_prefill[r] += n_new
            else:
                assert start == prompt[r] + got_decode[r] and got_prefill[r] == prompt[r]
                got_decode[r] += 1
        S.apply_iteration(entries, prompt, prefilled, gen_len, generated, state)
    assert state == [S.FINISHED] * n
    assert got_prefill == prompt and got_decode == gen_len            # every token exactly once
    order = [first_seen[r] for r in range(n)]
    assert order == sorted(order)                                      # arrival order is kept
