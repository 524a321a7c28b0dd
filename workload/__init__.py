"""Seeded synthetic inputs for the co-serving layer iteration.

This package holds data definitions and random-input recipes only.  It contains
none of the method's arithmetic (no norm, projection, attention, LoRA or index-map
code): the CPU oracle and the HIP path each receive the same bytes from here and
compute everything else on their own.
"""
from .configs import LayerCfg, Request, CONFIGS, TARGETS, target_dims  # noqa: F401
from . import gen  # noqa: F401
