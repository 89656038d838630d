"""fp64 CPU oracle of the multi-stream decode-attention step -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares nothing with the HIP library (no headers, helpers or tables).
"""
from .pasta_oracle import (  # noqa: F401
    Geom,
    append,
    attention,
    attention_dense,
    attention_q64,
    build,
    elem_offset,
    gather_map,
    merge,
    num_threads,
    partial,
    phys_row,
    rope,
    round_pool,
    rows_per_layer,
    visible_dense,
    visible_events,
    widen_pool,
)
