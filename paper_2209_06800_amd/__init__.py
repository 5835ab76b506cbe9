"""MI355X-native hot path of MGG's full-graph GNN layer (arXiv 2209.06800).

``binding`` mirrors the C ABI of ``libmgg.so`` (``include/mgg.h``); ``inputs`` draws the
seeded synthetic workloads; ``build`` compiles the library for gfx950.
"""
from .binding import (  # noqa: F401
    MggError, Partition, mgg_aggregate, mgg_build_partition, mgg_get_option, mgg_layer_forward,
    mgg_layer_workspace_bytes, mgg_set_option, mgg_split_edge_balanced, mgg_time_aggregate, mgg_update,
    mgg_version,
)
