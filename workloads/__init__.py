"""Seeded synthetic inputs for the split-FFN path.

This package only *makes inputs*: shapes, random draws, the planted heavy set,
rounding of the draws to their storage dtype, and the remainder's low-rank
factor inputs.  It holds none of the method's arithmetic (no activation, no
score, no selection, no quantiser, no forward), imports neither the oracle nor
the HIP package, and is the one module both sides share.
"""
from .configs import CONFIGS, FFNConfig, get_config  # noqa: F401
from .gen import (  # noqa: F401
    bf16_round,
    fp16_round,
    make_layer,
    make_tokens,
    planted_set,
    storage_round,
    truncated_factors,
    gaussian_factors,
    remainder_order,
    make_factors,
    seed_for,
)
