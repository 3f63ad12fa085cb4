"""Batch -> virtual-node partition and combination weights.

Section 3.2: each batch is split among the virtual nodes; Section 5.1/5.2: the
nodes may have unequal sizes and node i's average gradient is weighted by
b_i / B so that every example counts once.
"""
import numpy as np


def partition(node_sizes, batch):
    """Returns (off int32 [V+1], w float32 [V]).

    Node i owns the contiguous rows off[i] .. off[i+1]-1 of the batch, in batch
    order.  w[i] is the single IEEE fp32 division float32(b_i) / float32(B).
    Raises ValueError when the sizes are not a partition of the batch."""
    sizes = [int(b) for b in node_sizes]
    if len(sizes) < 1:
        raise ValueError("need at least one virtual node")
    if any(b < 1 for b in sizes):
        raise ValueError("every virtual node needs at least one sample")
    if sum(sizes) != int(batch):
        raise ValueError("node sizes do not sum to the batch size")
    off = np.zeros(len(sizes) + 1, dtype=np.int32)
    for i, b in enumerate(sizes):
        off[i + 1] = off[i] + b
    w = np.array([np.float32(b) / np.float32(batch) for b in sizes], dtype=np.float32)
    return off, w


def node_of_sample(node_sizes, batch):
    """int32 [B]: index of the node that owns each batch row (plain loop)."""
    owner = np.empty(int(batch), dtype=np.int32)
    row = 0
    for i, b in enumerate(node_sizes):
        for _ in range(int(b)):
            owner[row] = i
            row += 1
    if row != int(batch):
        raise ValueError("node sizes do not sum to the batch size")
    return owner
