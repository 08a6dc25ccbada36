"""CPU oracle of the ConfLayers self-speculative-decoding hot path.

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg
may import this package.  It is written from the paper alone and shares no code with the
HIP library.
"""
from .decoder import OracleModel, argmax_lowest, round_bf16, round_fp16, confidence_from_logits, DEFAULT_CLAMP, DEFAULT_EPS
from .ssd import OracleSSD, generate_ssd, generate_vanilla
from .select_skip import SelectParams, select_skip, uniform_skip
from .search import SearchDriver

__all__ = ["OracleModel", "argmax_lowest", "round_bf16", "round_fp16", "confidence_from_logits", "DEFAULT_CLAMP", "DEFAULT_EPS",
           "OracleSSD", "generate_ssd", "generate_vanilla", "SelectParams", "select_skip",
           "uniform_skip", "SearchDriver"]
