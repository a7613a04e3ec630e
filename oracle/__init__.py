"""OScaR CPU oracle (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never imports it.
"""
from .oscar_ref import (  # noqa: F401
    F32, BF16, F16, ZP_INT, ZP_MIN, SCALE_NONE, SCALE_L2,
    OracleConfig, OracleCache, build_oracle, lib,
    fwht, key_transform, query_transform, quant_params, quant_code, dequant,
    quant_group, round_dtype, sumsq_tree, plain_attn, max_threads,
)
