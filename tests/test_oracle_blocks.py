"""Pins for oracle/blocks.py: brute force, the paper's two formulations, closed forms, pooling (CPU only)."""
import os
import numpy as np
import pytest

import oracle
from workloads import masks

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [tuple(int(x) for x in ln.split()) for ln in f if ln.strip() and not ln.startswith("#")]


def _rand_mask(seed, N, Mb=1):
    m = masks.random_blocks(128 * ((N + 127) // 128), seed, blk=16, p_empty=0.35, p_full=0.35)[0][:N, :N]
    out = np.stack([np.roll(m, 5 * i, axis=1) for i in range(Mb)])
    return (out * np.random.default_rng(seed).integers(1, 255, out.shape, dtype=np.uint8)).astype(np.uint8)


@pytest.mark.parametrize("N,Br,Bc", [(64, 16, 16), (96, 32, 16), (50, 16, 32), (200, 64, 64), (37, 8, 16)])
def test_counts_match_four_loop_brute_force(N, Br, Bc):
    mask = _rand_mask(N, N, Mb=2)
    cnt = oracle.block_counts(mask, Br, Bc)
    for m in range(2):
        assert np.array_equal(cnt[m], oracle.brute_block_counts(mask[m], Br, Bc))
    assert cnt.sum() == np.count_nonzero(mask)


@pytest.mark.parametrize("N,Br,Bc", [(64, 16, 16), (200, 64, 32), (50, 16, 32)])
def test_any_formulation_equals_sum_formulation(N, Br, Bc):
    """Sec. 4 defines BinBlkMat by 'any non-zero'; Appendix A's kernel by 'block sum > 0'."""
    mask = _rand_mask(N + 1, N)
    assert np.array_equal(oracle.bin_blk_mat(mask, Br, Bc), (oracle.block_counts(mask, Br, Bc) > 0).astype(np.uint8))
    cls = oracle.block_class(mask, Br, Bc)
    assert np.array_equal(cls != 0, oracle.bin_blk_mat(mask, Br, Bc) != 0)


def test_shape_follows_paper():
    for N, BI, BJ, r, c in _rows("bin_blk_mat_shape.txt"):
        assert (N // BI, N // BJ) == (r, c)
        m = np.zeros((1, N, N), dtype=np.uint8)
        assert oracle.block_class(m, BI, BJ).shape == (1, r, c)
    assert oracle.bin_blk_mat(np.zeros((1, 256, 256), dtype=np.uint8), 128, 32).shape == (1, 2, 8)


def test_padded_tail_block_is_never_full():
    mask = np.ones((1, 200, 200), dtype=np.uint8)
    cls = oracle.block_class(mask, 64, 64)[0]
    assert cls.shape == (4, 4)
    assert np.all(cls[:3, :3] == 2) and np.all(cls[3, :] == 1) and np.all(cls[:, 3] == 1)
    r = oracle.run_index(cls[None])
    assert list(r["total_ones"][0]) == [3, 3, 3, 0] and list(r["offset"][0]) == [0, 0, 0, 0]


def test_or_pooling_consistency():
    mask = _rand_mask(3, 256)
    fine = oracle.bin_blk_mat(mask, 16, 16)[0]
    coarse = oracle.bin_blk_mat(mask, 32, 32)[0]
    pooled = fine.reshape(8, 2, 8, 2).max(axis=(1, 3))
    assert np.array_equal(coarse, pooled)
    cf, cc = oracle.block_class(mask, 16, 16)[0], oracle.block_class(mask, 32, 32)[0]
    assert np.array_equal(cc == 2, (cf.reshape(8, 2, 8, 2) == 2).all(axis=(1, 3)))


def test_all_ones_closed_form():
    idx = oracle.block_index(masks.all_ones(256), 64, 32)
    assert np.all(idx["cls"] == 2) and np.all(idx["bin_blk_mat"] == 1)
    assert np.all(idx["offset"] == 0) and np.all(idx["total_ones"] == 8)
    assert np.all(idx["nz_lo"] == 0) and np.all(idx["nz_hi"] == 8) and np.all(idx["nz_cnt"] == 8)
    assert list(idx["row_ptr"][0]) == [0, 8, 16, 24, 32]
    assert np.array_equal(idx["col_idx"], np.tile(np.arange(8, dtype=np.uint32) | np.uint32(0x80000000), 4))


def test_causal_closed_form_square_tiles():
    idx = oracle.block_index(masks.causal(512), 64, 64)
    for i in range(8):
        assert list(idx["cls"][0, i]) == [2] * i + [1] + [0] * (7 - i)
        assert (idx["offset"][0, i], idx["total_ones"][0, i]) == (0, i)
        assert (idx["nz_lo"][0, i], idx["nz_hi"][0, i], idx["nz_cnt"][0, i]) == (0, i + 1, i + 1)


def test_causal_closed_form_paper_tile_128x32():
    idx = oracle.block_index(masks.causal(1024), 128, 32)
    for i in range(8):
        assert idx["total_ones"][0, i] == 4 * i and idx["offset"][0, i] == 0
        assert idx["nz_cnt"][0, i] == 4 * i + 4
        assert list(idx["cls"][0, i, 4 * i:4 * i + 4]) == [1, 1, 1, 1]


def test_sliding_window_closed_form():
    # |i-j| <= 64 with 32x32 tiles: block (i,j) is full iff |i-j| <= 1, partial iff |i-j| in {2, 3}... derive:
    # full iff max |r-c| over the block = 32|i-j| + 31 <= 64 -> |i-j| <= 1; non-empty iff 32|i-j| - 31 <= 64 -> |i-j| <= 2
    N, w = 512, 64
    idx = oracle.block_index(masks.sliding_window(N, w), 32, 32)
    nb = N // 32
    for i in range(nb):
        lo, hi = max(0, i - 2), min(nb, i + 3)
        assert (idx["nz_lo"][0, i], idx["nz_hi"][0, i]) == (lo, hi)
        flo, fhi = max(0, i - 1), min(nb, i + 2)
        assert (idx["offset"][0, i], idx["total_ones"][0, i]) == (flo, fhi - flo)


def test_longest_run_leftmost_tie_and_noncontiguous_rows():
    cls = np.array([[[2, 2, 0, 2, 2, 1, 0],
                     [1, 2, 0, 2, 2, 2, 0],
                     [0, 0, 0, 0, 0, 0, 0],
                     [0, 1, 0, 0, 0, 2, 0]]], dtype=np.uint8)
    r = oracle.run_index(cls)
    assert list(r["offset"][0]) == [0, 3, 0, 5]
    assert list(r["total_ones"][0]) == [2, 3, 0, 1]
    assert list(r["nz_lo"][0]) == [0, 0, 0, 1]
    assert list(r["nz_hi"][0]) == [6, 6, 0, 6]
    assert list(r["nz_cnt"][0]) == [5, 5, 0, 2]
    rp, ci = oracle.sparse_index(cls)
    assert list(rp[0]) == [0, 5, 10, 10, 12]
    F = 0x80000000
    assert list(ci[:12]) == [0 | F, 1 | F, 3 | F, 4 | F, 5, 0, 1 | F, 3 | F, 4 | F, 5 | F, 1, 5 | F]


def test_sparse_index_planes_have_fixed_capacity():
    cls = np.zeros((2, 2, 3), dtype=np.uint8)
    cls[0, 1, 2] = 1
    cls[1, 0, 0] = 2
    cls[1, 1, 1] = 1
    rp, ci = oracle.sparse_index(cls)
    assert rp.tolist() == [[0, 0, 1], [0, 1, 2]]
    assert ci[0] == 2 and ci[6] == 0x80000000 and ci[7] == 1 and ci.size == 12


def test_column_index_hand_example_and_plane_capacity():
    cls = np.array([[[2, 2, 0, 2],
                     [1, 2, 0, 0],
                     [0, 1, 0, 2]]], dtype=np.uint8)
    cp, ri = oracle.column_index(cls)
    F = 0x80000000
    assert cp.tolist() == [[0, 2, 5, 5, 7]]
    assert list(ri[:7]) == [0 | F, 1, 0 | F, 1 | F, 2, 0 | F, 2 | F] and ri.size == 12
    two = np.stack([cls[0], cls[0][::-1]])
    cp2, ri2 = oracle.column_index(two)
    assert cp2[1].tolist() == [0, 2, 5, 5, 7] and list(ri2[12:19]) == [1, 2 | F, 0, 1 | F, 2 | F, 0 | F, 2 | F]


def test_column_index_rebuilds_the_class_matrix_and_mirrors_the_row_list():
    rng = np.random.default_rng(5)
    cls = rng.integers(0, 3, size=(2, 7, 5)).astype(np.uint8)
    cls[0, :, 2] = 0                                   # an empty column
    cp, ri = oracle.column_index(cls)
    back = np.zeros_like(cls)
    for m in range(2):
        for j in range(5):
            ent = ri[m * 35 + cp[m, j]: m * 35 + cp[m, j + 1]]
            rows = (ent & 0x7fffffff).astype(np.int64)
            assert np.all(np.diff(rows) > 0)
            back[m, rows, j] = np.where(ent >> 31, 2, 1)
    assert np.array_equal(back, cls)
    # the column list of a matrix is the row list of its transpose
    rp, ci = oracle.sparse_index(np.ascontiguousarray(cls.transpose(0, 2, 1)))
    assert np.array_equal(rp, cp) and np.array_equal(ci, ri)


@pytest.mark.parametrize("N", [64, 200, 130])
def test_packed_bits_roundtrip(N):
    mask = _rand_mask(N + 7, N, Mb=2)
    pk = oracle.packed_bits(mask)
    W = -(-N // 64)
    assert pk.shape == (2, W, N) and pk.dtype == np.uint64
    # independent unpacking route: bytes -> bits, little-endian
    by = pk.view(np.uint8).reshape(2, W, N, 8)
    bits = np.unpackbits(by, axis=-1, bitorder="little")              # [Mb, W, N, 64]
    full = bits.transpose(0, 2, 1, 3).reshape(2, N, W * 64)
    assert np.array_equal(full[:, :, :N], (mask != 0).astype(np.uint8))
    assert not full[:, :, N:].any()


def test_skip_rule_matches_paper_wording():
    """Sec. 4: the element mask is read only for visited blocks before `offset` or past the run of
    `total_ones` blocks; every block inside [offset, offset+total_ones) must be all ones."""
    mask = masks.packed_sequences(512, 1, 5, mu=4.0, hi=128)
    idx = oracle.block_index(mask, 32, 32)
    cnt = oracle.block_counts(mask, 32, 32)
    for i in range(16):
        o, t = idx["offset"][0, i], idx["total_ones"][0, i]
        assert np.all(cnt[0, i, o:o + t] == 32 * 32)
        for j in range(16):
            inside = o <= j < o + t
            if idx["bin_blk_mat"][0, i, j] and not inside and idx["cls"][0, i, j] == 2:
                assert t >= 1            # a full block outside the run exists only if a longer/equal run was kept


def _fake_lists(rp, width):
    """A col_idx array whose entry at position p of plane m is the recognisable value 1000*m + p (bit 31 set on odd p)."""
    Mb = rp.shape[0]
    ci = np.zeros((Mb, width), dtype=np.uint32)
    for m in range(Mb):
        for p in range(int(rp[m, -1])):
            ci[m, p] = (1000 * m + p) | (0x80000000 if p % 2 else 0)
    return ci.reshape(-1)


def _sched(rows, width=512):
    rp = np.array(rows, dtype=np.int32)
    return oracle.schedule(rp, _fake_lists(rp, width))


def test_schedule_cuts_only_long_rows():
    # rows with 3, 0, 40, 5 entries: mean of non-empty = 16 -> T = 32 -> only the 40-entry row is cut, into 2 x 20;
    # the last int of a part is the list entry at its first position (position 23 is odd: bit 31 set -> negative)
    s = _sched([[0, 3, 3, 43, 48]])
    assert (s[0], s[1], s[2]) == (2, 32, 1) and not s[3:8].any()
    assert s[8:24].reshape(2, 8).tolist() == [[2, 3, 20, 0, 2, 0, 0, 3 - 2**31], [2, 23, 20, 1, 2, 0, 0, 23 - 2**31]]
    # the floor of the threshold: rows of 1, 33 -> mean 17 -> T = 34: nothing cut; rows 1, 1, 1, 40 -> T = 32: 40 cut
    assert _sched([[0, 1, 34]])[:3].tolist() == [0, 34, 0]
    assert _sched([[0, 1, 2, 3, 43]])[:3].tolist() == [2, 32, 1]
    assert _sched([[0, 5, 10, 15]])[0] == 0          # uniform rows: nothing cut
    # row records (row, first position, entries, first entry) in launch order.  Up to 4 rows are one group: rows by
    # length, longest first: lengths 3, 0, 40, 5 -> rows 2, 3, 0, 1; an empty row has first entry -1; equal lengths ->
    # higher row first (causal masks: last row first)
    assert s[-16:].reshape(4, 4).tolist() == [[2, 3, 40, 3 - 2**31], [3, 43, 5, 43 - 2**31], [0, 0, 3, 0], [1, 3, 0, -1]]
    s2 = _sched([[0, 5, 10, 15], [0, 1, 3, 6]])
    assert s2[-24:].reshape(6, 4).tolist() == [[2, 10, 5, 10], [1, 5, 5, 5 - 2**31], [0, 0, 5, 0],
                                              [2, 3, 3, 1003 - 2**31], [1, 1, 2, 1001 - 2**31], [0, 0, 1, 1000]]


def test_schedule_launch_order_groups_of_four_rows():
    # 11 rows: groups {0..3}, {4..7}, {8..10} whose longest rows have 2, 30, 5 entries -> groups 1, 2, 0; inside group 1
    # the 30-entry row 6 first, then the equal rows from the highest down
    lens = [2] * 4 + [1] * 4 + [5] * 3
    lens[6] = 30
    rp = np.zeros((1, 12), dtype=np.int32)
    rp[0, 1:] = np.cumsum(lens)
    s = oracle.schedule(rp, _fake_lists(rp, 128))
    order = s[-4 * 11:].reshape(11, 4)
    assert order[:, 0].tolist() == [6, 7, 5, 4, 10, 9, 8, 3, 2, 1, 0]
    assert all(order[k, 1] == rp[0, order[k, 0]] and order[k, 2] == lens[order[k, 0]] for k in range(11))
    lens2 = [1] * 8                                        # two groups with equal longest rows: the higher rows first
    rp2 = np.zeros((1, 9), dtype=np.int32)
    rp2[0, 1:] = np.cumsum(lens2)
    assert oracle.schedule(rp2, _fake_lists(rp2, 32))[-32:].reshape(8, 4)[:, 0].tolist() == list(range(7, -1, -1))
    # the longest row decides, not the total: group {0..3} = 9 + 1 + 1 + 1 goes before group {4..7} = 4 x 8
    rp3 = np.zeros((1, 9), dtype=np.int32)
    rp3[0, 1:] = np.cumsum([9, 1, 1, 1, 8, 8, 8, 8])
    assert oracle.schedule(rp3, _fake_lists(rp3, 64))[-32:].reshape(8, 4)[:, 0].tolist() == [0, 3, 2, 1, 7, 6, 5, 4]
    # long rows (mean 30 -> T = 60 > 32): no grouping, plain longest-first order
    rp4 = np.zeros((1, 7), dtype=np.int32)
    rp4[0, 1:] = np.cumsum([40, 10, 30, 20, 50, 30])
    s4 = oracle.schedule(rp4, _fake_lists(rp4, 256))
    assert s4[1] == 60 and s4[-24:].reshape(6, 4)[:, 0].tolist() == [4, 0, 5, 2, 3, 1]


def test_schedule_parts_tile_each_cut_row_exactly():
    rng = np.random.default_rng(0)
    counts = rng.integers(0, 300, size=(3, 37))
    counts[rng.random(counts.shape) < 0.6] //= 20
    rp = np.zeros((3, 38), dtype=np.int32)
    rp[:, 1:] = np.cumsum(counts, axis=1)
    lists = _fake_lists(rp, 37 * 300)
    s = oracle.schedule(rp, lists)
    nparts, T, ncut = int(s[0]), int(s[1]), int(s[2])
    assert T == max(32, 2 * -(-int(counts.sum()) // int((counts > 0).sum())))
    parts = s[8:8 + 8 * nparts].reshape(nparts, 8)
    covered = np.zeros(counts.shape, dtype=np.int64)
    for q, (r, first, nt, k, np_, qf, rho, e_first) in enumerate(parts):
        m, i = divmod(int(r), 37)
        assert (int(e_first) & 0xffffffff) == int(lists.reshape(3, -1)[m, first])
        assert counts[m, i] > T and np_ == -(-counts[m, i] // T) and 1 <= nt <= T and q == qf + k
        assert first == rp[m, i] + covered[m, i]            # parts are consecutive slices of the row's list
        covered[m, i] += nt
    cut = counts > T
    assert np.array_equal(covered[cut], counts[cut]) and not covered[~cut].any()
    assert ncut == int(cut.sum()) and nparts <= counts.size          # the bound the workspace size relies on
    assert sorted(set(parts[:, 6].tolist())) == list(range(ncut))


def test_column_schedule_hand_example_and_tiling():
    # columns with 3, 0, 40, 5 entries: mean of non-empty = 16 -> T = 32 -> the 40-entry column is cut into 2 x 20
    cp = np.array([[0, 3, 3, 43, 48]], dtype=np.int32)
    s = oracle.column_schedule(cp, _fake_lists(cp, 512))
    assert (s[0], s[1], s[2]) == (2, 32, 1) and not s[3:8].any() and s.size == 8 + 12 * 4
    assert s[8:24].reshape(2, 8).tolist() == [[2, 3, 20, 0, 2, 0, 0, 3 - 2**31], [2, 23, 20, 1, 2, 0, 0, 23 - 2**31]]
    # launch order: longest column first; records (column, first position, entries, first entry), -1 for an empty one
    assert s[-16:].reshape(4, 4).tolist() == [[2, 3, 40, 3 - 2**31], [3, 43, 5, 43 - 2**31], [0, 0, 3, 0], [1, 3, 0, -1]]
    # equal lengths: the higher column first; every plane on its own
    cpe = np.array([[0, 2, 4, 5, 7], [0, 1, 1, 1, 4]], dtype=np.int32)
    se = oracle.column_schedule(cpe, _fake_lists(cpe, 16))
    assert se[-32:].reshape(8, 4)[:, 0].tolist() == [3, 1, 0, 2, 3, 0, 2, 1]
    assert se[-32:].reshape(8, 4)[4].tolist() == [3, 1, 3, 1001 - 2**31] and se[-4:].tolist() == [1, 1, 0, -1]
    # the floor of the threshold is 16 here: columns of 1, 1, 1, 20 -> mean 6 -> T = 16 -> 20 is cut into 2 x 10
    cp2 = np.array([[0, 1, 2, 3, 23]], dtype=np.int32)
    s2 = oracle.column_schedule(cp2, _fake_lists(cp2, 64))
    assert s2[:3].tolist() == [2, 16, 1] and s2[8:24].reshape(2, 8)[:, :5].tolist() == [[3, 3, 10, 0, 2], [3, 13, 10, 1, 2]]
    rng = np.random.default_rng(1)
    counts = rng.integers(0, 200, size=(2, 29))
    counts[rng.random(counts.shape) < 0.7] //= 25
    cp3 = np.zeros((2, 30), dtype=np.int32)
    cp3[:, 1:] = np.cumsum(counts, axis=1)
    lists = _fake_lists(cp3, 29 * 200)
    s3 = oracle.column_schedule(cp3, lists)
    nparts, T, ncut = int(s3[0]), int(s3[1]), int(s3[2])
    assert T == max(16, 2 * -(-int(counts.sum()) // int((counts > 0).sum())))
    covered = np.zeros(counts.shape, dtype=np.int64)
    for q, (c, first, nt, k, np_, qf, rho, e_first) in enumerate(s3[8:8 + 8 * nparts].reshape(nparts, 8)):
        m, j = divmod(int(c), 29)
        assert (int(e_first) & 0xffffffff) == int(lists.reshape(2, -1)[m, first])
        assert counts[m, j] > T and np_ == -(-counts[m, j] // T) and 1 <= nt <= T and q == qf + k
        assert first == cp3[m, j] + covered[m, j]
        covered[m, j] += nt
    cut = counts > T
    assert np.array_equal(covered[cut], counts[cut]) and not covered[~cut].any()
    assert ncut == int(cut.sum()) and nparts <= counts.size


def test_rectangular_mask_blocks_index_and_packed_bits():
    rng = np.random.default_rng(9)
    mask = (rng.random((2, 70, 200)) < 0.3).astype(np.uint8)
    mask[0, :64, 64:128] = 1
    mask[1, :, 128:] = 0
    cnt = oracle.block_counts(mask, 64, 64)
    assert cnt.shape == (2, 2, 4)
    for m in range(2):
        assert np.array_equal(cnt[m], oracle.brute_block_counts(mask[m], 64, 64))
    cls = oracle.block_class(mask, 64, 64)
    assert cls[0, 0, 1] == 2 and np.all(cls[1, :, 2:] == 0) and cls[0, 1, 1] == 1       # the ragged block row is never full
    assert np.array_equal(oracle.bin_blk_mat(mask, 64, 64), (cls != 0).astype(np.uint8))
    pk = oracle.packed_bits(mask)
    assert pk.shape == (2, 4, 70)
    bits = np.unpackbits(pk.view(np.uint8).reshape(2, 4, 70, 8), axis=-1, bitorder="little").reshape(2, 4, 70, 64)
    back = bits.transpose(0, 2, 1, 3).reshape(2, 70, 256)[:, :, :200]
    assert np.array_equal(back, mask) and not bits.transpose(0, 2, 1, 3).reshape(2, 70, 256)[:, :, 200:].any()
    idx = oracle.block_index(mask, 64, 64)
    assert idx["row_ptr"].shape == (2, 3) and idx["col_ptr"].shape == (2, 5)
