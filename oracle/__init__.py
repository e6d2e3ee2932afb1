"""fp64 CPU oracle for GQA decode attention.

Test infrastructure only: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports it and it
never imports the product package.
"""
from .gqa_oracle import (build_oracle, causal_attn_rows, decode_attn, kv_append, shared_prefix_attn,  # noqa: F401
                         OracleResult)
