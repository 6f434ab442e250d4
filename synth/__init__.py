"""Seeded synthetic inputs: model shapes, random-init weights, prompts and
forced-acceptance schedules.  Used by both the CPU oracle's tests and the GPU
library's tests and benchmark; holds none of the method's arithmetic.
"""
from .configs import ModelShape, PairConfig, PAIRS, pair, shrink  # noqa: F401
from .weights import make_weights, make_pair_weights, quantize_rows, quantize_weights, to_numpy_weights  # noqa: F401
from .prompts import make_prompts  # noqa: F401
from .alpha import alpha_constant, alpha_piecewise  # noqa: F401
from .kv import make_kv  # noqa: F401
