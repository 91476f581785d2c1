"""fp64 CPU oracle for SWA + sink attention.  TEST INFRASTRUCTURE ONLY.

Nothing on the product path may import this package: only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` do.
It shares no code with ``paper_2512_10411_amd`` and never imports it.
"""
from .swaa_oracle import (  # noqa: F401
    build_oracle,
    decode_elems,
    input_format,
    oracle_num_threads,
    swaa_attn_bwd_oracle,
    swaa_attn_oracle,
    swaa_attn_oracle_numpy,
    swaa_decode_oracle,
    swaa_decode_oracle_numpy,
)
