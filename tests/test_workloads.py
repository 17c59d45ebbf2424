"""The synthetic workload generators: determinism, structure and the paper's tree-size formula (CPU only)."""
import os
import numpy as np

from workloads import masks, make_config, small_variant, f32_to_bf16_bits, CONFIGS
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_medusa_tree_size_formula_matches_paper_example():
    with open(os.path.join(GOLD, "medusa_tree_mask_size.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    for K, s, size in rows:
        assert masks.medusa_tree_size([int(s)] * int(K)) == int(size)
    assert masks.medusa_tree_size([10, 5, 3, 2]) == 10 + 50 + 150 + 300
    assert len(masks.full_tree_parents([4, 4, 4, 4])) == 340


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]                 # ties
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(f32_to_bf16_bits(x), want)


def test_generators_are_deterministic():
    a, b = make_config("C1"), make_config("C1")
    for key in ("mask", "q", "k", "v"):
        assert np.array_equal(a[key], b[key])


def test_tiny_config_structure():
    c = make_config("C1")
    m = c["mask"][0]
    assert m.shape == (256, 256) and np.all(np.diag(m) == 1) and set(np.unique(m)) <= {0, 1}


def test_packed_mask_is_block_diagonal_causal():
    c = small_variant("C2", N=512, B=2, H=1, with_qkv=False)
    m = c["mask"]
    assert m.shape == (2, 512, 512)
    assert not np.triu(m[0], 1).any()
    pad_rows = np.flatnonzero(m[0].sum(1) == 0)
    assert pad_rows.size == 0 or pad_rows[0] + pad_rows.size == 512   # padding is a suffix
    assert not np.array_equal(m[0], m[1])


def test_tree_mask_structure():
    par = masks.random_subtree([10, 5, 3, 2], 256, 3)
    assert len(par) == 256 and np.all(par < np.arange(256)) and (par == -1).sum() <= 10
    m = masks.tree_verification(64, par)[0]
    assert np.all(m[64:, :64] == 1) and np.all(np.diag(m) == 1) and not np.triu(m, 1).any()
    t = 200
    anc = []
    a = t
    while a >= 0:
        anc.append(a)
        a = par[a]
    assert sorted(np.flatnonzero(m[64 + t, 64:])) == sorted(anc)


def test_longctx_mask_structure():
    m = masks.longctx_sparse(2048, 1, window=256, n_global=32, n_rand=2)[0]
    assert np.all(m[:32] == 1) and np.all(m[:, :32] == 1)
    i = np.arange(2048)
    band = np.abs(i[:, None] - i[None, :]) <= 128
    assert np.all(m[band] == 1)


def test_graph_mask_is_symmetric_with_self_loops_and_rcm_reduces_blocks():
    N = 2048
    a = small_variant("C5", N=N, with_qkv=False)["mask"][0]
    assert np.array_equal(a, a.T) and np.all(np.diag(a) == 1)
    kw = dict(xm=max(2.0, 84.0 * N / 32768 * 4), cap=max(16, int(2000 * N / 32768 * 4)))
    seed = small_variant("C5", N=64, with_qkv=False)["seed"]
    s = masks.graph_mask(N, seed, reorder="none", **kw)[0]
    assert np.array_equal(masks.graph_mask(N, seed, reorder="rcm", **kw)[0], a)
    assert s.sum() == a.sum()
    nb = N // 64
    blocks = lambda m: m.reshape(nb, 64, nb, 64).any(axis=(1, 3)).mean()
    assert blocks(a) < 0.6 * blocks(s)


def test_config_table_matches_stated_shapes():
    assert CONFIGS["C2"] == dict(B=4, H=16, N=4096, d=64, Mb=4, family="packed")
    assert CONFIGS["C3"]["N"] == 1024 + 256 and CONFIGS["C3"]["d"] == 128
    assert CONFIGS["C4"]["N"] == 16384 and CONFIGS["C5"]["N"] == 32768


def test_further_mask_families_of_the_evaluation():
    """Input-bidirectional packing, plain and dilated windows (paper Sec. 5, ALPACA and Longformer masks)."""
    m = masks.packed_sequences(512, 1, 5, bidirectional_prefix=0.4, mu=np.log(40.0), hi=128)[0]
    lens = masks.packed_lengths(512, 5, mu=np.log(40.0), hi=128)
    pos = 0
    for L in lens:
        p = int(round(0.4 * L))
        blk = m[pos:pos + L, pos:pos + L]
        assert np.all(blk[:p, :p] == 1)                              # inputs see each other
        assert np.array_equal(blk[p:], np.tril(np.ones((L, L), dtype=np.uint8))[p:])   # outputs: causal over the sequence
        assert not blk[:p, p:].any()                                 # inputs do not see outputs
        assert not m[pos:pos + L, :pos].any() and not m[pos:pos + L, pos + L:].any()
        pos += L
    assert not m[pos:].any()
    w = masks.sliding_window(100, 7)[0]
    d = masks.dilated_window(100, 7, 2)[0]
    assert np.array_equal(masks.dilated_window(100, 7, 1)[0], w)
    assert w[50].sum() == 15 and d[50].sum() == 15 and d[50, 36] == 1 and d[50, 37] == 0 and d[50, 64] == 1 and d[50, 66] == 0
    assert np.array_equal(d, d.T) and np.all(np.diag(d) == 1)
    for name in ("C2b", "C4w", "C4d"):
        cfg = small_variant(name, N=512, B=1, H=1, with_qkv=False)
        assert cfg["mask"].shape[1:] == (512, 512) and cfg["mask"].any()
