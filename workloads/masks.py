"""Seeded attention-mask generators shaped like the paper's workloads (Sec. 5: MEDUSA tree masks,
packed fine-tuning masks, Longformer-style sparse masks; Sec. 4: RCM-reordered sparse masks).

Every function returns uint8 arrays with values in {0, 1}; element [.., i, j] != 0 means query i may
attend to key j.  Shape is [Mb, N, N] (Mb = number of distinct masks in the batch).
"""
import numpy as np


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def all_ones(N: int) -> np.ndarray:
    return np.ones((1, N, N), dtype=np.uint8)


def causal(N: int) -> np.ndarray:
    return np.tril(np.ones((N, N), dtype=np.uint8))[None]


def sliding_window(N: int, w: int) -> np.ndarray:
    """|i - j| <= w."""
    i = np.arange(N)
    return (np.abs(i[:, None] - i[None, :]) <= w).astype(np.uint8)[None]


def dilated_window(N: int, w: int, dilation: int) -> np.ndarray:
    """Longformer's dilated sliding window: |i - j| <= w * dilation and (i - j) divisible by the dilation, i.e. w keys
    on each side with gaps of dilation - 1 between them (dilation = 1 is sliding_window)."""
    i = np.arange(N)
    diff = i[:, None] - i[None, :]
    return ((np.abs(diff) <= w * dilation) & (diff % dilation == 0)).astype(np.uint8)[None]


def random_blocks(N: int, seed: int, blk: int = 64, p_empty=0.4, p_full=0.3, p_elem=0.5) -> np.ndarray:
    """Grid of blk x blk blocks, each empty / full / partial (Bernoulli(p_elem) per element); diagonal forced on."""
    assert N % blk == 0
    rng = _rng(seed)
    nb = N // blk
    kind = rng.choice(3, size=(nb, nb), p=[p_empty, p_full, 1.0 - p_empty - p_full])
    m = np.zeros((N, N), dtype=np.uint8)
    for bi in range(nb):
        for bj in range(nb):
            sl = (slice(bi * blk, (bi + 1) * blk), slice(bj * blk, (bj + 1) * blk))
            if kind[bi, bj] == 1:
                m[sl] = 1
            elif kind[bi, bj] == 2:
                m[sl] = (rng.random((blk, blk)) < p_elem).astype(np.uint8)
    m[np.arange(N), np.arange(N)] = 1
    return m[None]


def random_elements(N: int, seed: int, p: float = 0.5, empty_rows=()) -> np.ndarray:
    """Unstructured Bernoulli(p) mask; rows listed in empty_rows are cleared."""
    rng = _rng(seed)
    m = (rng.random((N, N)) < p).astype(np.uint8)
    for r in empty_rows:
        m[r, :] = 0
    return m[None]


def packed_lengths(N: int, seed: int, mu=5.3, sigma=0.7, lo=16, hi=1024):
    """Sequence lengths ~ round(lognormal(mu, sigma)) clipped to [lo, hi], appended while they fit in N."""
    rng = _rng(seed)
    lens, pos = [], 0
    while True:
        L = int(np.clip(np.rint(rng.lognormal(mu, sigma)), lo, hi))
        if pos + L > N:
            break
        lens.append(L)
        pos += L
    return lens


def packed_sequences(N: int, Mb: int, seed: int, bidirectional_prefix: float = 0.0, **kw) -> np.ndarray:
    """Block-diagonal causal mask per packed sequence; rows/cols after the last sequence are all zero
    (padding).  With bidirectional_prefix = f > 0 the first round(f*L) tokens of every sequence attend to
    each other in both directions (the paper's "Input-Bidirectional" packing)."""
    out = np.zeros((Mb, N, N), dtype=np.uint8)
    for m in range(Mb):
        pos = 0
        for L in packed_lengths(N, seed + 7919 * m, **kw):
            blk = np.tril(np.ones((L, L), dtype=np.uint8))
            p = int(round(bidirectional_prefix * L))
            if p > 0:
                blk[:p, :p] = 1
            out[m, pos:pos + L, pos:pos + L] = blk
            pos += L
    return out


def medusa_tree_size(s) -> int:
    """Number of nodes of the full candidate tree with per-level branching s[0], s[1], ...: sum_k prod_{i<=k} s_i."""
    total, prod = 0, 1
    for sk in s:
        prod *= int(sk)
        total += prod
    return total


def full_tree_parents(s):
    """Parent index (-1 for first-level nodes) of every node of the full tree, nodes numbered in level order."""
    parents, level_start, level_size = [], 0, 1
    prev_nodes = [-1]
    for sk in s:
        cur = []
        for p in prev_nodes:
            for _ in range(sk):
                cur.append(len(parents))
                parents.append(p)
        prev_nodes = cur
    return np.asarray(parents, dtype=np.int64)


def random_subtree(s, n_nodes: int, seed: int):
    """Random ancestor-closed subset of the full tree with n_nodes nodes: start empty, repeatedly add a
    uniformly random frontier node (a node whose parent is present, or a first-level node).  Returns the
    parent array of the subset re-indexed in level order (-1 = child of the prefix root)."""
    parents = full_tree_parents(s)
    total = len(parents)
    assert n_nodes <= total
    rng = _rng(seed)
    children = [[] for _ in range(total)]
    roots = []
    for v, p in enumerate(parents):
        (roots if p < 0 else children[p]).append(v)
    chosen = np.zeros(total, dtype=bool)
    frontier = list(roots)
    for _ in range(n_nodes):
        k = int(rng.integers(len(frontier)))
        v = frontier[k]
        frontier[k] = frontier[-1]
        frontier.pop()
        chosen[v] = True
        frontier.extend(children[v])
    keep = np.flatnonzero(chosen)            # level order is preserved by ascending node id
    new_id = -np.ones(total, dtype=np.int64)
    new_id[keep] = np.arange(len(keep))
    return np.where(parents[keep] < 0, -1, new_id[np.maximum(parents[keep], 0)])


def tree_verification(prefix: int, tree_parents: np.ndarray) -> np.ndarray:
    """Causal prefix followed by tree tokens; tree token t attends to the whole prefix, its ancestors and itself."""
    T = len(tree_parents)
    N = prefix + T
    m = np.zeros((N, N), dtype=np.uint8)
    m[:prefix, :prefix] = np.tril(np.ones((prefix, prefix), dtype=np.uint8))
    m[prefix:, :prefix] = 1
    for t in range(T):
        a = t
        while a >= 0:
            m[prefix + t, prefix + a] = 1
            a = int(tree_parents[a])
    return m[None]


def longctx_sparse(N: int, seed: int, window: int = 512, n_global: int = 64, n_rand: int = 3, blk: int = 64) -> np.ndarray:
    """Sliding window |i-j| <= window/2, union n_global global tokens (full rows and columns), union n_rand
    distinct random blk-wide key blocks (fully on) per blk-row query block."""
    assert N % blk == 0
    rng = _rng(seed)
    nb = N // blk
    m = np.zeros((N, N), dtype=np.uint8)
    half = window // 2
    i = np.arange(N)
    for r0 in range(0, N, 1024):                      # banded fill in row chunks to bound temporaries
        r1 = min(N, r0 + 1024)
        c0, c1 = max(0, r0 - half), min(N, r1 + half)
        m[r0:r1, c0:c1] = (np.abs(i[r0:r1, None] - i[None, c0:c1]) <= half)
    m[:n_global, :] = 1
    m[:, :n_global] = 1
    for bi in range(nb):
        for bj in rng.choice(nb, size=min(n_rand, nb), replace=False):
            m[bi * blk:(bi + 1) * blk, bj * blk:(bj + 1) * blk] = 1
    return m[None]


def locality_graph_edges(N: int, seed: int, xm: float = 84.0, shape: float = 1.5, cap: int = 2000, min_reach: int = 8):
    """Directed edge draws of a power-law graph with latent 1-D locality: node i draws
    h_i = min(cap, xm*(1+Pareto(shape))) neighbours uniformly from [i - r_i, i + r_i], r_i = max(h_i, min_reach)."""
    rng = _rng(seed)
    h = np.minimum(cap, np.floor(xm * (1.0 + rng.pareto(shape, size=N)))).astype(np.int64)
    h = np.minimum(h, N - 1)
    src = np.repeat(np.arange(N, dtype=np.int64), h)
    reach = np.repeat(np.maximum(h, min_reach), h)
    off = np.floor((rng.random(src.size) * 2.0 - 1.0) * (reach + 1)).astype(np.int64)
    dst = np.clip(src + off, 0, N - 1)
    return src, dst


def graph_mask(N: int, seed: int, reorder: str = "rcm", **kw) -> np.ndarray:
    """Symmetric power-law graph with self loops.  The node labels are scrambled by a random permutation
    (an unstructured input); reorder = "rcm" then applies reverse Cuthill-McKee, "none" leaves it scrambled."""
    import scipy.sparse as sp
    from scipy.sparse.csgraph import reverse_cuthill_mckee
    src, dst = locality_graph_edges(N, seed, **kw)
    rng = _rng(seed + 1)
    scramble = rng.permutation(N)
    src, dst = scramble[src], scramble[dst]
    rows = np.concatenate([src, dst, np.arange(N)])
    cols = np.concatenate([dst, src, np.arange(N)])
    A = sp.csr_matrix((np.ones(rows.size, dtype=np.uint8), (rows, cols)), shape=(N, N))
    A.data[:] = 1
    if reorder == "rcm":
        perm = np.asarray(reverse_cuthill_mckee(A, symmetric_mode=True), dtype=np.int64)
        inv = np.empty(N, dtype=np.int64)
        inv[perm] = np.arange(N)
        coo = A.tocoo()
        r, c = inv[coo.row], inv[coo.col]
    elif reorder == "none":
        coo = A.tocoo()
        r, c = coo.row, coo.col
    else:
        raise ValueError(reorder)
    m = np.zeros((N, N), dtype=np.uint8)
    m[r, c] = 1
    return m[None]
