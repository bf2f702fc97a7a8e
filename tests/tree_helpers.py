"""Checker-side tree helpers: written for the tests, independent of both the HIP path
and the oracle, so that a pin which uses them checks the oracle against something
other than itself."""
import numpy as np


def node_depths(parent) -> np.ndarray:
    """Number of nodes on each node's root path (a root counts 1), by a forward sweep."""
    d = np.zeros(len(parent), dtype=np.int32)
    for i, p in enumerate(parent):
        d[i] = 1 if p < 0 else d[p] + 1
    return d


def spec_tree(parent) -> np.ndarray:
    """Sec. 3.2.2, decode stage: the n drafted nodes followed by one appended token per
    node; appended token k (index n + k) is placed after node k's root path."""
    n = len(parent)
    return np.concatenate([np.asarray(parent, np.int32), np.arange(n, dtype=np.int32)])
