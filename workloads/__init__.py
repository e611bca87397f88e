"""Seeded synthetic inputs for the TokenCarve compression path.

This package only draws random numbers and shapes them like the paper's
workload (LLaVA-1.5 prefill: system tokens, a 24x24 grid of visual tokens,
prompt tokens).  It contains none of the method's arithmetic (no softmax, no
SVD, no scoring, no merging) and is the only code shared by the CPU oracle's
tests and the GPU path's tests.
"""
from .configs import CONFIGS, Workload, get_config  # noqa: F401
from .generate import (  # noqa: F401
    make_image,
    make_batch,
    planted_lowrank,
    round_to_storage,
)
