"""Slow, plain CPU reference for the certified-decode hot path.

Test infrastructure only: imported by tests/, the smoke check and the bench's
cpu_baseline leg.  The product path (the HIP library and its Python binding)
never imports this package, and this package never imports the product path.
"""
from .attention import (FLAG_ANY, FLAG_KEY, FLAG_PRECOND, FLAG_RANK, FLAG_TOTAL, FLAG_VAL,
                        RUNG_SHIFT, Tolerances, certified_head, key_term, softmax_attention)
from .cache import OracleLayerCache, ladder_decision
from . import quantizer
from . import adaptive
from .adaptive import SelectorParams

__all__ = ["FLAG_ANY", "FLAG_KEY", "FLAG_PRECOND", "FLAG_RANK", "FLAG_TOTAL", "FLAG_VAL",
           "RUNG_SHIFT", "Tolerances", "certified_head", "key_term", "softmax_attention",
           "OracleLayerCache", "ladder_decision", "quantizer", "adaptive", "SelectorParams"]
