"""CPU oracle for the token-level co-serving layer iteration (FlexLLM, arXiv 2402.18789).

TEST INFRASTRUCTURE ONLY.  Plain numpy, fp64 by default, no blocking, fusion or
reordering beyond what the definitions state.  Nothing in the product path may
import this package: only the tests, the smoke check and the benchmark's
cpu_baseline leg do.  It shares no code with the HIP library.

Modules
  maps.py   index maps of a mixed token batch (integer, exact)
  ops.py    per-operator definitions (RMSNorm, RoPE, SwiGLU, causal attention, LoRA)
            and their hand-derived backward rules
  layer.py  one decoder layer: whole-sequence forward/backward (the definition),
            the cache-based mixed-batch forward and the token-window backward
            (Algorithm 2), and the multi-layer drivers
  prune.py  static graph pruning (Algorithm 1) on an operator graph

Pins: see tests/test_oracle_*.py.  Every function here is pinned by at least one
test that does not call the function itself to produce the expected value, except
where the header of a function says "parity unpinned".
"""
