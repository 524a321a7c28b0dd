"""Host-side parity of the hybrid token scheduler (Sec. 6.2) through the C ABI: window sizes and
iteration entries are integers and must equal the oracle's exactly; the latency estimate that decides
the window is computed in double on both sides, in the same order, and must be bit-identical."""
import numpy as np
import pytest

import paper_2402_18789_amd.binding as B
from oracle import sched as S
from workload import gen


def random_model(seed, n_c, n_s, monotone):
    g = gen.rng(seed, "schedhost", "model", n_c, n_s, monotone)
    c_grid = np.cumsum(g.integers(1, 300, n_c)).astype(np.int32) - 1
    s_grid = np.concatenate([[0], np.cumsum(g.integers(1, 200, n_s - 1))]).astype(np.int32)
    ms = (g.random((n_c, n_s)) * 5).astype(np.float32)
    if monotone:
        ms = np.cumsum(np.cumsum(ms, axis=0), axis=1).astype(np.float32)
    return c_grid, s_grid, ms


@pytest.mark.parametrize("seed,n_c,n_s,monotone", [(0, 2, 2, True), (1, 5, 6, True), (2, 7, 3, False), (3, 3, 9, False)])
def test_estimate_and_window_equal_the_oracle(seed, n_c, n_s, monotone):
    c_grid, s_grid, ms = random_model(seed, n_c, n_s, monotone)
    model = B.HostLatencyModel(c_grid, s_grid, ms)
    cg, sg, table = c_grid.tolist(), s_grid.tolist(), [[float(v) for v in row] for row in ms]
    g = gen.rng(seed, "schedhost", "queries")
    lo, hi = float(ms.min()), float(ms.max())
    for _ in range(400):
        c = int(g.integers(0, int(c_grid[-1]) * 2 + 2))
        s = int(g.integers(0, int(s_grid[-1]) * 2 + 2))
        want = S.latency_estimate(cg, sg, table, c, s)
        got = B.flexco_latency_estimate(model, c, s)
        assert got == want, (c, s)                                   # bit-identical doubles
        slo = float(g.uniform(lo - 1.0, hi * 1.5))
        s_avail = int(g.integers(0, int(s_grid[-1]) * 2 + 2))
        quantum = int(g.choice([1, 7, 16, 64]))
        assert B.flexco_sched_window(model, c, slo, s_avail, quantum) == S.pick_window(cg, sg, table, c, slo, s_avail, quantum)


def test_window_with_the_slo_exactly_on_a_grid_value():
    c_grid, s_grid = np.array([0, 100], np.int32), np.array([0, 64, 128], np.int32)
    ms = np.array([[1.0, 2.0, 4.0], [1.0, 2.0, 4.0]], np.float32)
    model = B.HostLatencyModel(c_grid, s_grid, ms)
    assert B.flexco_sched_window(model, 50, 2.0, 128, 64) == 64     # f = SLO counts as met
    assert B.flexco_sched_window(model, 50, 1.999, 128, 64) == 0
    assert B.flexco_sched_window(model, 50, 4.0, 100, 64) == 100    # s_avail itself, between grid points: f = 3.125


@pytest.mark.parametrize("seed,max_batch,budget,chunk", [(0, 4, 64, 16), (1, 8, 32, 32), (2, 1, 7, 3), (3, 16, 256, 64),
                                                         (4, 64, 1024, 256)])
def test_inference_stage_equals_the_oracle_iteration_by_iteration(seed, max_batch, budget, chunk):
    g = gen.rng(seed, "schedhost", "stream")
    n = 60
    prompt = g.integers(1, 400, n).astype(np.int32)
    gen_len = g.integers(0, 40, n).astype(np.int32)
    c_state = {"prefilled": np.zeros(n, np.int32), "generated": np.zeros(n, np.int32), "state": np.zeros(n, np.int32)}
    o_prefilled, o_generated, o_state = [0] * n, [0] * n, [S.WAITING] * n
    for it in range(100000):
        want = S.schedule_inference(prompt.tolist(), o_prefilled, gen_len.tolist(), o_generated, o_state, max_batch, budget, chunk)
        got, c = B.flexco_sched_inference(prompt, c_state["prefilled"], gen_len, c_state["generated"], c_state["state"],
                                          max_batch, budget, chunk)
        assert [tuple(int(x) for x in e) for e in got] == want, it
        assert c == sum(e[3] for e in want)
        assert c_state["state"].tolist() == o_state
        if not want:
            break
        S.apply_iteration(want, prompt.tolist(), o_prefilled, gen_len.tolist(), o_generated, o_state)
        B.flexco_sched_advance(got, prompt, c_state["prefilled"], gen_len, c_state["generated"], c_state["state"])
        assert c_state["prefilled"].tolist() == o_prefilled and c_state["generated"].tolist() == o_generated
        assert c_state["state"].tolist() == o_state
    assert o_state == [S.FINISHED] * n


def test_scheduler_error_paths():
    c_grid, s_grid = np.array([0, 100], np.int32), np.array([0, 64], np.int32)
    ms = np.ones((2, 2), np.float32)
    model = B.HostLatencyModel(c_grid, s_grid, ms)
    with pytest.raises(B.FlexcoError):
        B.flexco_sched_window(model, 10, 1.0, 64, 0)                 # quantum
    with pytest.raises(B.FlexcoError):
        B.flexco_sched_window(model, 10, 1.0, -1, 16)                # s_avail
    bad = B.HostLatencyModel(np.array([5, 5], np.int32), s_grid, ms)  # grid does not ascend
    with pytest.raises(B.FlexcoError):
        B.flexco_latency_estimate(bad, 1, 1)
    one = np.ones(1, np.int32)
    with pytest.raises(B.FlexcoError):                                # progress beyond the prompt
        B.flexco_sched_inference(one, one * 2, one, one * 0, one * 0, 4, 16, 8)
    with pytest.raises(B.FlexcoError):
        B.flexco_sched_inference(one, one * 0, one, one * 0, one * 0, 0, 16, 8)
