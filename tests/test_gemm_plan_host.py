"""The projection kernels' launch plan (flexco_gemm_plan: host arithmetic, no GPU): the plans of the configurations'
own products are what the measurements chose, and any plan is well formed - its launches cover the output columns
exactly once with tile shapes the kernel is built for, K splits cut K into whole 64-wide stages and fit the scratch."""
import numpy as np
import pytest

import paper_2402_18789_amd.binding as B
from workload import CONFIGS

pytestmark = pytest.mark.skipif(B.HOST_ONLY, reason="needs the whole library, this is a host-only build")

SPLITK_COLS = 32768          # floats of split-K scratch per row that the layer calls bring


def proj_shapes(cfg):
    qkv = cfg.q_dim + 2 * cfg.kv_dim
    return {"qkv": (qkv, cfg.hidden), "o": (cfg.hidden, cfg.q_dim), "gate_up": (2 * cfg.ffn, cfg.hidden),
            "down": (cfg.hidden, cfg.ffn)}


def test_forward_plans_of_the_benchmark_step():
    cfg = CONFIGS["c2_llama8b_layer"]
    sh = proj_shapes(cfg)
    T = 1024
    plan = {k: B.flexco_gemm_plan(T, n, kk, 0, 0) for k, (n, kk) in sh.items()}
    assert plan["qkv"] == [(128, 192, 6144, 1, 4)]                                    # 256 tiles: one round
    assert plan["o"] == [(128, 128, 4096, 1, 4)] and plan["down"] == [(128, 128, 4096, 1, 4)]
    # one round of 256 x 256 tiles and one of 256 x 192 tiles side by side
    assert plan["gate_up"] == [(256, 256, 16384, 1, 2), (256, 192, 12288, 1, 2)]


def test_input_gradient_plans_by_window_length():
    c2, c4 = CONFIGS["c2_llama8b_layer"], CONFIGS["c4_qwen14b_full"]
    # a 256-row window: two row tiles of 128, K cut so that every block slot pulls on the weight stream
    for (n, kk), splits in (((c2.ffn, c2.hidden), 2), ((c2.hidden, 2 * c2.ffn), 8), ((c2.q_dim, c2.hidden), 8)):
        assert B.flexco_gemm_plan(256, n, kk, 1, 256 * SPLITK_COLS) == [(128, 128, n, splits, 2)]
    # 1024 rows at the 14B shape: the large tile where few of them still fill the chip (down: 216 tiles; gate/up: 80 x 3),
    # the small one for the output and q/k/v products (80 large tiles would leave 96 CUs idle)
    pe = 1024 * SPLITK_COLS
    assert B.flexco_gemm_plan(1024, c4.ffn, c4.hidden, 1, pe) == [(256, 256, c4.ffn, 1, 2)]
    assert B.flexco_gemm_plan(1024, c4.hidden, 2 * c4.ffn, 1, pe) == [(256, 256, c4.hidden, 3, 2)]
    assert B.flexco_gemm_plan(1024, c4.q_dim, c4.hidden, 1, pe) == [(128, 128, c4.q_dim, 4, 2)]
    assert B.flexco_gemm_plan(1024, c4.hidden, c4.q_dim + 2 * c4.kv_dim, 1, pe) == [(128, 128, c4.hidden, 4, 2)]
    # without scratch K stays whole
    assert B.flexco_gemm_plan(1024, c4.hidden, 2 * c4.ffn, 1, 0)[0][3] == 1
    assert B.flexco_gemm_plan(256, c2.hidden, 2 * c2.ffn, 1, 0) == [(128, 128, c2.hidden, 1, 2)]


def test_decode_only_batches_cut_k():
    c2 = CONFIGS["c2_llama8b_layer"]
    (bm, bn, cols, splits, stages), = B.flexco_gemm_plan(16, c2.q_dim + 2 * c2.kv_dim, c2.hidden, 0, 16 * SPLITK_COLS)
    assert (bm, bn, cols) == (128, 128, 6144) and splits > 1
    assert B.flexco_gemm_plan(16, 6144, c2.hidden, 0, 0) == [(128, 128, 6144, 1, 4)]   # no scratch, no cut


def test_any_plan_is_well_formed():
    g = np.random.default_rng(7)
    shapes = {(128, 128), (128, 192), (256, 192), (256, 256)}
    for _ in range(3000):
        M = int(g.integers(1, 5000))
        N = 8 * int(g.integers(1, 8000))
        K = 64 * int(g.integers(1, 900))
        trans = int(g.integers(0, 2))
        pe = int(g.choice([0, M * SPLITK_COLS, 1 << 20]))
        plan = B.flexco_gemm_plan(M, N, K, trans, pe)
        assert 1 <= len(plan) <= 2, (M, N, K, trans, pe, plan)
        assert sum(p[2] for p in plan) == N
        for i, (bm, bn, cols, splits, stages) in enumerate(plan):
            assert (bm, bn) in shapes and cols > 0 and stages in (2, 4)
            if trans:
                assert (bm, bn) in ((128, 128), (256, 256)) and len(plan) == 1
            if i + 1 < len(plan):
                assert cols % bn == 0                       # the next launch starts at a tile boundary
            assert splits >= 1 and K % (64 * splits) == 0
            if splits > 1:
                assert splits * M * N <= pe and len(plan) == 1
                assert K // splits >= 4 * 64


def test_rejects_shapes_the_matrix_core_path_does_not_take():
    for args in ((0, 64, 64, 0, 0), (64, 64, 64, 0, -1)):
        with pytest.raises(B.FlexcoError):
            B.flexco_gemm_plan(*args)
    for args in ((64, 64, 72, 0, 0), (64, 12, 64, 1, 0)):
        with pytest.raises(B.FlexcoError):
            B.flexco_gemm_plan(*args)
