"""Seeded synthetic input generators for the swap-executor hot path.

This package produces *inputs only*: operator strings, tensor lifetime tables,
alloc/free event lists, arena placements and configuration-given swap sets.  It
holds none of the method's arithmetic (no tokenisation, no timeline scan, no
matching, no policy timing): both the CPU oracle and the HIP library consume
what is generated here and each computes the method on its own.

The five workload configurations mirror the shapes of the paper's LLM training
runs (a stacked-decoder Llama-like model, Sec. 4.1 and Sec. 6.1); no dataset,
weights or recorded traces are involved.
"""
from .layouts import (OP_DT, EVENT_DT, TENSOR_DT, ANCHOR_DT, POLICY_DT, DESC_DT,
                      ACTION_DT, NONE_OP, DT_BF16, DT_FP32, DT_U8,
                      PH_FWD, PH_BWD, PH_OPT)
from .rng import SplitMix64
from .transformer import Trace, ModelShape, build_trace, config_shape, config_swap_set
from .small_tensor import build_small_tensor_stress
from .arena import place_first_fit, ArenaPlan

__all__ = [n for n in dir() if not n.startswith("_")]
