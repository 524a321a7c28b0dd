"""flexco: one co-serving iteration of a LoRA-augmented decoder layer over a mixed token
batch (FlexLLM, arXiv 2402.18789), as hand-written HIP kernels for MI355X behind a C ABI.

`binding` mirrors include/flexco.h one to one; `host` owns device memory for callers that
use PyTorch tensors.  Importing fails if libflexco.so has not been built: there is no
fallback path.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
