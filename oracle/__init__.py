"""CPU oracle of the GNS hot path -- test infrastructure only.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The HIP library never does.
"""
from .gns_oracle import (  # noqa: F401
    UNIFORM, CACHE_ONLY, CACHE_FIRST, W_PRINTED, W_UNBIASED,
    build_oracle, philox4x32_10, cache_draw_node, sample_cache, floyd,
    p_cache, edge_weight, sample_layer, walk_weights, build_block, sample_blocks,
    gather, aggregate, sage_dense, OracleBlock,
)
