"""Draft-tree bookkeeping of tree-structured drafting (Sec. 4.1), test infrastructure only: what the
library's tree plan and parent arrays are compared with.  Plain Python, no dependency on the GPU package."""
from __future__ import annotations

import numpy as np


def tree_batch_sizes(tree):
    """Batch size at each draft position of a tree (N_1..N_gamma): every node at position i - 1 has
    N_i children, so B_i = N_1 * ... * N_i (Sec. 4.1)."""
    sizes, b = [], 1
    for n in tree:
        b *= int(n)
        sizes.append(b)
    return sizes


def tree_parents(tree):
    """Parent-index arrays of a tree (N_1..N_gamma) grown from one root: the N_i children of node p
    at position i sit in slots p*N_i .. p*N_i + N_i - 1, so parent[j] = j // N_i."""
    return [np.arange(b, dtype=np.int32) // np.int32(n)
            for b, n in zip(tree_batch_sizes(tree), tree)]
