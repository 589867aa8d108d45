"""Seeded node-to-partition maps for the partitioned (several-GPU) execution of a computation graph.

Input manufacture only: which partition stores which node.  None of the method's arithmetic lives here.
"""
from __future__ import annotations

import numpy as np


def hash_partition(n_nodes: int, n_part: int, seed: int = 1005) -> np.ndarray:
    """Random-hash partitioning (the paper's default placement, Sec. 7): every node gets a partition drawn
    uniformly and independently of the graph.  int32 [n_nodes]."""
    rng = np.random.Generator(np.random.PCG64([seed, 7]))
    return rng.integers(0, n_part, size=n_nodes, dtype=np.int32)


def block_partition(n_nodes: int, n_part: int) -> np.ndarray:
    """Contiguous id ranges of equal size (what a locality-aware partitioner gives on a graph whose ids
    follow its communities).  int32 [n_nodes]."""
    return (np.arange(n_nodes, dtype=np.int64) * n_part // max(n_nodes, 1)).astype(np.int32)
