"""CPU oracle for the MoIN hot path -- test infrastructure only.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library.
"""
from .oracle import (  # noqa: F401
    AdapterCache,
    build,
    dist2,
    histogram,
    kmeans_update,
    lora_linear,
    lora_linear_mx,
    max_threads,
    merge_adapters,
    mx_dequantize,
    mx_quantize,
    retain_clusters,
    route,
    route_topk,
    slot_map,
)
