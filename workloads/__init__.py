"""Seeded synthetic inputs shared by the tests, the bench and the CPU oracle.

This package only *draws data* (values, context lengths, placements).  It holds none of
the attention / placement arithmetic: neither the HIP library nor the oracle lives here,
and neither of them imports the other.
"""
from .synth import (  # noqa: F401
    Workload,
    gen_kv,
    gen_q,
    gen_q_steps,
    gen_kv_new,
    gen_rising_k,
    make_workload,
    normal_bf16_table,
    pack_bitmap,
)
