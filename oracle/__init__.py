"""CPU oracle for the FlowMM KV-cache merge (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.
"""
from .flowmm_oracle import (  # noqa: F401
    build, score, flow, select, match, merge, merge_weighted, decode_attention, round_output, layer_pass, num_threads,
    cache_append, cache_remerge,
)
