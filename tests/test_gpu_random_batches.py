"""Seeded random mixed batches through the whole layer path (forward over several co-serving iterations, then
the token-window backward) against the oracle: random numbers of decode / prefill requests, context lengths,
chunk and window lengths that are not multiples of any tile, random key splits, every head grouping the
kernels special-case.  Each case is a pure function of its seed."""
import numpy as np
import pytest

from workload import gen
from test_gpu_parity import C1, SMALL_BF16, SMALL_BF16_G5, SMALL_BF16_MHA, SMALL_BF16_G8, run_layer_case, say

pytestmark = pytest.mark.gpu

# tensors that miss 2e-2 against the plain oracle and are held to 5e-3 against the storage-rounding oracle, per seed
STORAGE_EXCEPTIONS = {}

CFGS = [SMALL_BF16, SMALL_BF16_G5, SMALL_BF16_MHA, SMALL_BF16_G8, C1]


@pytest.mark.parametrize("seed", range(20))
def test_random_mixed_batch(seed):
    g = gen.rng(seed, "random_batches")
    cfg = CFGS[seed % len(CFGS)]
    n_dec = int(g.integers(0, 13))
    ctx = g.integers(1, 301, size=n_dec)
    prefill = []
    for _ in range(int(g.integers(0, 3))):
        total = int(g.integers(2, 200))
        start = int(g.integers(0, total - 1))
        prefill.append((start, int(g.integers(1, total - start + 1)), total))
    L = int(g.integers(1, 181))
    ft_window = int(g.integers(max(1, L // 6), L + 1))       # at most about six forward iterations
    first = min(ft_window, L)
    batch = gen.mixed_batch(16, seed, decode_ctx=ctx, prefill=prefill, finetune=[(0, first, L)], extra_capacity=8)
    # backward windows: a random composition of L
    bwd, left = [], L
    while left > 0:
        s = int(g.integers(1, left + 1))
        bwd.append(s)
        left -= s
    split = int(g.choice([0, 2, 4, 8]))
    need_dx = bool(g.integers(0, 2)) or not any(t in cfg.lora_targets for t in ("q", "k", "v"))
    say(f"random batch {seed}: {cfg.name}, {n_dec} decode, prefill {prefill}, finetune L={L} windows of {ft_window}, "
        f"backward {bwd}, split {split}, need_dx {need_dx}")
    run_layer_case(cfg, batch, ft_window=ft_window, prefill_chunk=int(g.integers(1, 80)), bwd_windows=bwd, seed=seed,
                   split=split, need_dx=need_dx, storage_exceptions=STORAGE_EXCEPTIONS.get(seed, ()))
