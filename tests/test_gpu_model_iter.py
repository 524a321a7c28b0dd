"""The whole-model iteration driver (forward through every layer, loss head, backward through every
layer, Adam) runs and leaves finite results; the numbers of the same calls chained over layers are
checked against the oracle in test_gpu_train.py and test_gpu_parity.py."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_model_iteration_two_layers():
    from paper_2402_18789_amd import model_iter
    say("model iteration, 2 layers of the 8B shape, vocabulary 4096")
    r = model_iter.run(n_layers=2, steps=1, warmup=1, vocab=4096)
    say(str({k: r[k] for k in ("ms_per_iteration", "forward_ms", "loss_head_ms", "backward_ms", "loss", "lora_grad_norm_dB")}))
    assert r["finite"]
    assert r["config"]["tokens"] == 2048 and r["config"]["finetune_tokens"] == 512
    # a random head's loss over the window's rows, scaled by window / sequence: ln(V) / 4 to a few percent
    import math
    assert abs(r["loss"] - math.log(4096) * 512 / 2048) < 0.2 * math.log(4096) * 512 / 2048
    assert r["lora_grad_norm_dB"] > 0
    assert r["forward_ms"] > 0 and r["backward_ms"] > 0
