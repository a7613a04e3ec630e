"""OScaR CPU oracle (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never imports it.
"""
from .oscar_ref import (  # noqa: F401
    F32, BF16, F16, ZP_INT, ZP_MIN, SCALE_NONE, SCALE_L2, SCALE_MAX, SCALE_MEAN_ABS, NORM_PER_HEAD, NORM_ALL_KV_HEADS,
    OracleConfig, OracleCache, build_oracle, lib,
    fwht, key_transform, query_transform, token_norm_all_heads, key_transform_given_norm, quant_params, quant_code, dequant,
    quant_group, round_dtype, round_meta, sumsq_tree, sumabs_tree, plain_attn, max_threads,
)
