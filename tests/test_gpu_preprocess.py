"""GPU parity: block classes, BinBlkMat, packed bits, run index and sparse list, bit-exact against the oracle."""
import numpy as np
import pytest
import torch

from workloads import masks, small_variant, make_config
from gpu_util import index_to_numpy, assert_index_equal

pytestmark = pytest.mark.gpu


def _bbm():
    import paper_2409_15097_amd as bbm
    return bbm


def _run(mask_np, Br, Bc, row_stride=None, fused=True):
    bbm = _bbm()
    Mb, N, _ = mask_np.shape
    if row_stride is None:
        mask = torch.from_numpy(mask_np).cuda()
    else:
        buf = torch.zeros((Mb, N, row_stride), dtype=torch.uint8, device="cuda")
        buf[:, :, :N] = torch.from_numpy(mask_np).cuda()
        mask = buf[:, :, :N]
    idx = bbm.build_index(mask, Br, Bc, fused=fused)      # one-call entry point, or runs and list separately
    torch.cuda.synchronize()
    return idx


CASES = [
    ("C1", 256, 64, 64), ("C1", 256, 128, 64), ("C1", 256, 128, 32), ("C1", 256, 32, 128), ("C1", 256, 256, 256),
    ("C2", 1024, 128, 64), ("C2", 1024, 64, 64), ("C3", 640, 128, 64), ("C3", 640, 64, 16),
    ("C4", 2048, 128, 64), ("C4", 2048, 64, 64), ("C5", 2048, 128, 64), ("C5", 2048, 64, 64),
    ("C0d", 512, 128, 64), ("C0c", 512, 128, 64), ("C0c", 1024, 128, 32),
]


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("name,N,Br,Bc", CASES)
def test_index_bit_exact_small_variants(name, N, Br, Bc, fused):
    cfg = small_variant(name, N=N, B=2, H=1, with_qkv=False)
    idx = _run(cfg["mask"], Br, Bc, fused=fused)
    assert_index_equal(index_to_numpy(idx), cfg["mask"], Br, Bc)


@pytest.mark.parametrize("N,Br,Bc", [(200, 64, 64), (333, 128, 64), (1000, 128, 64), (77, 64, 64), (1, 64, 64),
                                     (1025, 100, 32), (2100, 7, 16), (64, 1, 64)])
def test_index_bit_exact_ragged_sizes(N, Br, Bc):
    rng = np.random.default_rng(N)
    blk = masks.random_blocks(64 * (-(-N // 64)), N, blk=32, p_empty=0.35, p_full=0.4)[0][:N, :N]
    mask = (blk * rng.integers(1, 255, blk.shape, dtype=np.uint8)).astype(np.uint8)[None]
    idx = _run(mask, Br, Bc)                       # rows not 16-byte aligned unless N % 16 == 0: byte path
    assert_index_equal(index_to_numpy(idx), mask, Br, Bc)
    stride = 16 * (-(-N // 16)) + 16
    idx = _run(mask, Br, Bc, row_stride=stride, fused=False)    # padded, aligned rows: vector path with a ragged tail
    assert_index_equal(index_to_numpy(idx), mask, Br, Bc)


def test_all_zero_and_all_ones_masks():
    for fill in (0, 1):
        mask = np.full((2, 320, 320), fill, dtype=np.uint8)
        idx = _run(mask, 64, 64)
        assert_index_equal(index_to_numpy(idx), mask, 64, 64)


def test_long_rows_of_blocks_cross_ballot_chunks():
    """nbc > 64 so that runs and lists span several 64-block ballot chunks."""
    N, Bc = 2304, 16                                # nbc = 144
    mask = np.zeros((1, N, N), dtype=np.uint8)
    mask[0, :64, 16 * 10:16 * 140] = 1              # one run crossing two chunk boundaries
    mask[0, 64:128, :16 * 64] = 1                   # run ending exactly at a chunk boundary
    mask[0, 64:128, 16 * 64 + 5] = 1                # followed by a partial block
    mask[0, 128:192, 16 * 63:16 * 65] = 1           # two-block run straddling the boundary
    mask[0, 128:192, 16 * 100:16 * 102] = 1         # equal-length run later: leftmost must win
    mask[0, 192:256, 16 * 128:] = 1                 # run reaching the row end
    for fused in (True, False):
        idx = _run(mask, 64, Bc, fused=fused)      # 36 rows x 3 chunks: still one launch when fused
        assert_index_equal(index_to_numpy(idx), mask, 64, Bc)


def test_more_block_rows_than_the_schedule_sorts():
    """Br = 1 gives 4200 block rows (> 4096): the schedule lists them from the last row to the first, unsorted."""
    N = 4200
    rng = np.random.default_rng(5)
    mask = (rng.random((1, N, N)) < 0.002).astype(np.uint8)
    mask[0, 100:110] = 1                            # a few full-width rows: long lists that the schedule cuts
    mask[0, 3000:3003, ::2] = 1
    for fused in (True, False):
        idx = _run(mask, 1, 64, fused=fused)
        got = index_to_numpy(idx)
        assert_index_equal(got, mask, 1, 64)
        assert got["sched"][0] > 0                  # parts exist
        assert np.array_equal(got["sched"][-4 * N:].reshape(N, 4)[:, 0], np.arange(N - 1, -1, -1))


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5"])
def test_index_bit_exact_full_size(name):
    cfg = make_config(name, with_qkv=False)
    for Br in (128, 64):
        idx = _run(cfg["mask"], Br, 64, fused=(Br == 128))
        assert_index_equal(index_to_numpy(idx), cfg["mask"], Br, 64)
        del idx


@pytest.mark.parametrize("Mb,N,Br,kind", [(3, 6000, 64, "window"), (2, 9000, 128, "packed"), (1, 14000, 128, "graph"), (5, 3333, 32, "window"),
                                          (2, 8192, 64, "blocks"), (1, 12000, 128, "window")])
def test_mid_size_class_matrices_list_and_schedule_in_one_launch(Mb, N, Br, kind):
    """More than 256 (block row, chunk) pairs and at most 1024 block rows per plane: the one-call index stage takes the
    general path, whose second launch fills the lists and writes the schedule.  Short rows (ranked in groups of four),
    long rows (ranked singly), rows the schedule cuts, several planes; the two-call stage runs the separate kernels."""
    rng = np.random.default_rng(N + Br)
    i, j = np.arange(N)[:, None], np.arange(N)[None, :]
    mask = np.zeros((Mb, N, N), dtype=np.uint8)
    for m in range(Mb):
        if kind == "window":
            mask[m] = np.abs(i - j) <= 100 + 150 * m
            mask[m, rng.integers(0, N, 5)] = 1                      # global queries: rows the schedule cuts
            mask[m][:, rng.integers(0, N, 5)] = 1                   # global keys
        elif kind == "packed":
            edges = np.sort(rng.integers(0, N, 40))
            seg = np.searchsorted(edges, np.arange(N))
            mask[m] = (seg[:, None] == seg[None, :]) & (j <= i)
        elif kind == "graph":
            mask[m] = (rng.random((N, N)) < 0.0005) | (np.abs(i - j) < 3)
            mask[m, 4000:4040] = 1
        else:
            cls = rng.choice(3, size=(-(-N // 64), -(-N // 64)), p=[0.7, 0.2, 0.1])
            blk = np.kron(cls, np.ones((64, 64), dtype=np.int64))[:N, :N]
            mask[m] = (blk == 1) | ((blk == 2) & (rng.random((N, N)) < 0.3))
    for fused in (True, False):
        idx = _run(mask, Br, 64, fused=fused)
        got = index_to_numpy(idx)
        assert_index_equal(got, mask, Br, 64)
    assert got["sched"][1] >= 32 and (kind != "window" or got["sched"][0] > 0)       # the window masks have cut rows
