"""Pins for oracle/reorder.py (CPU only): the textbook queue formulation, closed forms, invariants, a library routine."""
from collections import deque

import numpy as np
import scipy.sparse as sp
from scipy.sparse.csgraph import reverse_cuthill_mckee as scipy_rcm

import oracle
from workloads import masks


def _sym(N, seed, p):
    rng = np.random.default_rng(seed)
    a = rng.random((N, N)) < p
    a = a | a.T
    a[np.arange(N), np.arange(N)] = True
    return a.astype(np.uint8)


def _queue_cm(A):
    """Classical Cuthill-McKee with a queue: a dequeued node appends its unvisited neighbours by (degree, index)."""
    A = A != 0
    N = A.shape[0]
    deg = A.sum(axis=1)
    seen = np.zeros(N, dtype=bool)
    out = []
    while len(out) < N:
        start = min((int(deg[i]), i) for i in range(N) if not seen[i])[1]
        seen[start] = True
        q = deque([start])
        while q:
            u = q.popleft()
            out.append(u)
            for v in sorted((int(deg[v]), int(v)) for v in np.flatnonzero(A[u]) if not seen[v]):
                seen[v[1]] = True
                q.append(v[1])
    return np.asarray(out)


def test_level_formulation_equals_the_queue_algorithm():
    for seed, N, p in ((1, 40, 0.08), (2, 65, 0.04), (3, 30, 0.3), (4, 50, 0.01)):
        A = _sym(N, seed, p)
        assert np.array_equal(oracle.cuthill_mckee_order(A), _queue_cm(A)), seed


def test_result_is_a_permutation_also_with_isolated_nodes_and_several_components():
    A = np.zeros((12, 12), dtype=np.uint8)
    A[np.arange(12), np.arange(12)] = 1
    for i, j in ((0, 5), (5, 9), (2, 3), (3, 7), (7, 2)):
        A[i, j] = A[j, i] = 1
    perm = oracle.reverse_cuthill_mckee(A)
    assert sorted(perm.tolist()) == list(range(12))
    # isolated nodes (degree 1: the self loop) start first in Cuthill-McKee order, i.e. end up last after the reversal
    iso = [1, 4, 6, 8, 10, 11]
    assert perm[::-1][:6].tolist() == iso
    B = oracle.permute_mask(A, perm)
    assert np.array_equal(B, B.T) and B.sum() == A.sum() and oracle.bandwidth(B) <= 2


def test_scrambled_path_and_band_are_recovered():
    N = 50
    path = (np.abs(np.arange(N)[:, None] - np.arange(N)[None, :]) <= 1).astype(np.uint8)
    pi = np.random.default_rng(5).permutation(N)
    scrambled = path[pi][:, pi]
    assert oracle.bandwidth(scrambled) > 10
    perm = oracle.reverse_cuthill_mckee(scrambled)
    assert oracle.bandwidth(oracle.permute_mask(scrambled, perm)) == 1
    band = masks.sliding_window(64, 3)[0]              # a band is already optimal: the ordering must keep its width
    assert oracle.bandwidth(oracle.permute_mask(band, oracle.reverse_cuthill_mckee(band))) == 3


def test_bandwidth_is_comparable_to_the_library_routine():
    """Tie-breaking differs between implementations, so the orderings differ; the quality must not."""
    for seed in (6, 7, 8):
        N = 200
        base = (np.abs(np.arange(N)[:, None] - np.arange(N)[None, :]) <= 4) & (np.random.default_rng(seed).random((N, N)) < 0.6)
        base = (base | base.T).astype(np.uint8)
        base[np.arange(N), np.arange(N)] = 1
        pi = np.random.default_rng(seed + 10).permutation(N)
        A = base[pi][:, pi]
        ours = oracle.bandwidth(oracle.permute_mask(A, oracle.reverse_cuthill_mckee(A)))
        lib = np.asarray(scipy_rcm(sp.csr_matrix(A), symmetric_mode=True))
        theirs = oracle.bandwidth(A[lib][:, lib])
        assert ours <= oracle.bandwidth(A) // 4 and ours <= 2 * theirs + 2, (ours, theirs)


def test_reordering_reduces_the_non_zero_blocks_of_the_graph_workload():
    A = masks.graph_mask(1024, 3, reorder="none", xm=8.0, cap=60)[0]
    before = int((oracle.block_class(A[None], 64, 64) != 0).sum())
    B = oracle.permute_mask(A, oracle.reverse_cuthill_mckee(A))
    after = int((oracle.block_class(B[None], 64, 64) != 0).sum())
    assert after < before // 2, (before, after)


def test_joint_permutation_commutes_with_attention():
    """Attention on the reordered problem, un-permuted, is attention on the original problem."""
    rng = np.random.default_rng(9)
    N, d = 48, 8
    A = _sym(N, 9, 0.1)[None]
    q, k, v = (rng.standard_normal((1, 2, N, d)) for _ in range(3))
    perm = oracle.reverse_cuthill_mckee(A[0])
    O, lse = oracle.masked_attention(q, k, v, A)
    Op, lp = oracle.masked_attention(q[:, :, perm], k[:, :, perm], v[:, :, perm], oracle.permute_mask(A, perm))
    inv = np.argsort(perm)
    assert np.abs(Op[:, :, inv] - O).max() < 1e-12 and np.abs(lp[:, :, inv] - lse).max() < 1e-12


def test_hand_worked_example():
    """Edges 0-1, 0-2, 1-3, 2-3, 3-4 and self loops: degrees 3, 3, 3, 4, 2.  The walk starts at node 4 (minimum
    degree), reaches 3, then 1 and 2 (same parent, same degree: by index), then 0 (claimed by 1, the earlier parent)."""
    A = np.eye(5, dtype=np.uint8)
    for i, j in ((0, 1), (0, 2), (1, 3), (2, 3), (3, 4)):
        A[i, j] = A[j, i] = 1
    assert oracle.cuthill_mckee_order(A).tolist() == [4, 3, 1, 2, 0]
    assert oracle.reverse_cuthill_mckee(A).tolist() == [0, 2, 1, 3, 4]
    # a lower degree wins over a lower index inside a level: give node 2 a pendant neighbour 5
    B = np.eye(6, dtype=np.uint8)
    for i, j in ((0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (2, 5)):
        B[i, j] = B[j, i] = 1
    # degrees 3, 3, 4, 4, 2, 2: start 4 (degree 2, lower index than 5); 3; then 1 (degree 3) before 2 (degree 4);
    # then 0 (parent 1), then 5 (parent 2)
    assert oracle.cuthill_mckee_order(B).tolist() == [4, 3, 1, 2, 0, 5]
