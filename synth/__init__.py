"""Seeded synthetic inputs for the SRPE serving path.

This package only manufactures inputs: graphs, feature and embedding tables,
weights and query batches.  It contains none of the method's arithmetic (no
recompute-set selection, no aggregation, no layer math), so both the CPU oracle
and the GPU path can be fed from it without sharing any code of the method.
"""
from .graphs import power_law_graph, BaseGraph
from .tables import (normal_table, relu_normal_table, to_bf16_bits,
                     glorot, make_layers, LayerParams)
from .batches import make_batch, QueryBatch
from .configs import CONFIGS, Workload, build_workload
from .partition import hash_partition, block_partition
