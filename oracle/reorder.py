"""Oracle (test infrastructure): reverse Cuthill-McKee reordering of a sparse attention mask.

Paper Sec. 4 "Binary Block Masking with Reverse Cuthill-McKee (RCM)": the mask is treated as the adjacency matrix of a
graph and reordered so that its bandwidth shrinks and fewer blocks are non-zero.  The paper names the algorithm and
cites it; it fixes neither start nodes nor tie-breaking.  Readings fixed here (the published algorithm, with every
choice made deterministic):

* neighbours of node i = { j : mask[i, j] != 0 } (the mask is read row-wise; the method assumes a symmetric mask), the
  degree of i = their number (a self loop counts);
* each connected component is started at its unvisited node of minimum degree (ties: the smallest index), components
  in the order in which such nodes come up;
* breadth-first, level by level: the next level holds every unvisited neighbour of the current level, ordered by
  (position in the ordering of its earliest parent, degree, index) -- which is the classical queue formulation
  (each dequeued node appends its unvisited neighbours by increasing degree);
* the Cuthill-McKee ordering reversed is the result: perm[k] = the old index of the node placed at position k, and the
  reordered mask is mask[perm][:, perm].
"""
import numpy as np


def cuthill_mckee_order(mask2d):
    """mask2d [N, N] -> int64 [N]: the Cuthill-McKee ordering (not yet reversed), level by level."""
    A = np.asarray(mask2d) != 0
    N = A.shape[0]
    degree = A.sum(axis=1).astype(np.int64)
    visited = np.zeros(N, dtype=bool)
    order = []
    while len(order) < N:
        cand = np.flatnonzero(~visited)
        start = int(cand[np.lexsort((cand, degree[cand]))[0]])       # minimum degree, then smallest index
        visited[start] = True
        level_lo = len(order)
        order.append(start)
        while level_lo < len(order):
            level_hi = len(order)
            parent_pos = {}
            for pos in range(level_lo, level_hi):                      # earliest parent claims the node
                for v in np.flatnonzero(A[order[pos]] & ~visited):
                    parent_pos.setdefault(int(v), pos)
            nxt = sorted(parent_pos, key=lambda v: (parent_pos[v], degree[v], v))
            visited[nxt] = True
            order.extend(nxt)
            level_lo = level_hi
    return np.asarray(order, dtype=np.int64)


def reverse_cuthill_mckee(mask2d):
    """perm int64 [N]: perm[k] = old index of the node at new position k."""
    return cuthill_mckee_order(mask2d)[::-1].copy()


def permute_mask(mask, perm):
    """mask [Mb, N, N] (or [N, N]) reordered by perm on both axes."""
    mask = np.asarray(mask)
    if mask.ndim == 2:
        return mask[perm][:, perm]
    return np.stack([m[perm][:, perm] for m in mask])


def bandwidth(mask2d):
    """max |i - j| over the non-zero elements (0 for an empty mask)."""
    r, c = np.nonzero(mask2d)
    return int(np.abs(r - c).max()) if r.size else 0
