"""Exhaustive definition of the search result (TEST INFRASTRUCTURE).

The strategy search reaches exactly min_S t_o(G, D, S) (Thm. 1 and 2); the plain
definition of that value is Eq. 1 evaluated for every one of the C^N strategies.
Only usable on tiny graphs.
"""
from __future__ import annotations

import numpy as np


def all_costs(n_nodes, edges, C, tc, ts, tx) -> np.ndarray:
    """t_o for every strategy as an int64 array of shape (C,)*n_nodes (Eq. 1).

    Axis l is the configuration of node l.
    """
    if C ** n_nodes > (1 << 26):
        raise ValueError("too many strategies to enumerate")
    total = np.zeros((C,) * n_nodes, dtype=np.int64)
    for l in range(n_nodes):
        shape = [1] * n_nodes
        shape[l] = C
        total = total + (tc[l].astype(np.int64) + ts[l].astype(np.int64)).reshape(shape)
    for e, (i, j) in enumerate(np.asarray(edges).reshape(-1, 2)):
        i, j = int(i), int(j)
        shape = [1] * n_nodes
        shape[i] = C
        shape[j] = C
        t = tx[e].astype(np.int64)
        if i > j:                       # table is [src cfg][dst cfg]; axes are ordered by node id
            t = t.T
        total = total + t.reshape(shape)
    return total


def all_costs_ragged(n_nodes, edges, Cn, tc, ts, tx) -> np.ndarray:
    """Eq. 1 for every strategy when node l has Cn[l] configurations; tc, ts, tx concatenated."""
    Cn = [int(c) for c in Cn]
    if np.prod([float(c) for c in Cn]) > (1 << 26):
        raise ValueError("too many strategies to enumerate")
    tc, ts, tx = np.asarray(tc).reshape(-1), np.asarray(ts).reshape(-1), np.asarray(tx).reshape(-1)
    total = np.zeros(tuple(Cn), dtype=np.int64)
    off = 0
    for l in range(n_nodes):
        shape = [1] * n_nodes
        shape[l] = Cn[l]
        total = total + (tc[off:off + Cn[l]].astype(np.int64) + ts[off:off + Cn[l]].astype(np.int64)).reshape(shape)
        off += Cn[l]
    off = 0
    for i, j in np.asarray(edges).reshape(-1, 2):
        i, j = int(i), int(j)
        t = tx[off:off + Cn[i] * Cn[j]].astype(np.int64).reshape(Cn[i], Cn[j])
        off += Cn[i] * Cn[j]
        shape = [1] * n_nodes
        shape[i], shape[j] = Cn[i], Cn[j]
        if i > j:
            t = t.T
        total = total + t.reshape(shape)
    return total


def brute_force_ragged(n_nodes, edges, Cn, tc, ts, tx):
    total = all_costs_ragged(n_nodes, edges, Cn, tc, ts, tx)
    best = int(total.min())
    S = np.array(np.unravel_index(int(np.argmin(total)), total.shape), dtype=np.int32)
    return best, S, int((total == best).sum())


def brute_force(n_nodes, edges, C, tc, ts, tx):
    """(optimal cost, lexicographically lowest optimal strategy, number of optimal strategies)."""
    total = all_costs(n_nodes, edges, C, tc, ts, tx)
    best = int(total.min())
    flat = int(np.argmin(total))        # first occurrence in C order = node 0 most significant
    S = np.array(np.unravel_index(flat, total.shape), dtype=np.int32)
    return best, S, int((total == best).sum())
