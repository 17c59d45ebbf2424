"""GPU parity: reverse Cuthill-McKee ordering, mask permutation and row gathers against the oracle (bit-exact), and the
whole reordered pipeline against attention on the original problem."""
import numpy as np
import pytest
import torch

import oracle
from workloads import masks, make_qkv
from gpu_util import bf16_tensor, bf16_result_to_f64, assert_attention_close

pytestmark = pytest.mark.gpu


def _bbm():
    import paper_2409_15097_amd as bbm
    return bbm


def _sym(N, seed, p):
    rng = np.random.default_rng(seed)
    a = rng.random((N, N)) < p
    a = a | a.T
    a[np.arange(N), np.arange(N)] = True
    return a.astype(np.uint8)


def _cases():
    yield "random sparse", _sym(300, 1, 0.01)                       # several components, ragged N
    yield "random denser", _sym(130, 2, 0.1)
    path = (np.abs(np.arange(257)[:, None] - np.arange(257)[None, :]) <= 1).astype(np.uint8)
    pi = np.random.default_rng(3).permutation(257)
    yield "scrambled path", path[pi][:, pi]                         # 257 levels of one node
    iso = np.eye(100, dtype=np.uint8)
    iso[3, 70] = iso[70, 3] = 1
    yield "isolated nodes", iso                                      # 99 components
    star = np.eye(200, dtype=np.uint8)
    star[17, :] = 1
    star[:, 17] = 1
    yield "star", star                                               # one level of 199 nodes
    big = np.eye(5000, dtype=np.uint8)
    big[4321, :] = 1
    big[:, 4321] = 1
    big[np.arange(0, 4999, 2), np.arange(1, 5000, 2)] = 1                # unequal degrees among the 4999 nodes of the level
    big[np.arange(1, 5000, 2), np.arange(0, 4999, 2)] = 1
    yield "big star", big                                            # a level larger than one ranking sweep (4096 keys)
    yield "graph workload", masks.graph_mask(1024, 5, reorder="none", xm=8.0, cap=60)[0]
    yield "single node", np.ones((1, 1), dtype=np.uint8)
    yield "no self loops", (_sym(64, 4, 0.05) * (1 - np.eye(64, dtype=np.uint8))).astype(np.uint8)


@pytest.mark.parametrize("name,A", list(_cases()), ids=[n for n, _ in _cases()])
def test_rcm_order_matches_oracle(name, A):
    bbm = _bbm()
    print(f"rcm case {name} N={A.shape[0]}", flush=True)
    A = np.ascontiguousarray(A)
    perm = bbm.bbm_rcm_order(torch.from_numpy(A).cuda())
    torch.cuda.synchronize()
    want = oracle.reverse_cuthill_mckee(A)
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), want)


def test_rcm_order_with_a_padded_row_stride_and_unaligned_rows():
    bbm = _bbm()
    A = _sym(150, 6, 0.03)
    buf = torch.zeros((150, 173), dtype=torch.uint8, device="cuda")       # stride 173: the byte-wise path
    buf[:, :150] = torch.from_numpy(A).cuda()
    perm = bbm.bbm_rcm_order(buf[:, :150])
    torch.cuda.synchronize()
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), oracle.reverse_cuthill_mckee(A))


def test_permute_mask_and_gather_rows_match_numpy():
    bbm = _bbm()
    N = 333
    rng = np.random.default_rng(7)
    mask = (rng.random((2, N, N)) < 0.2).astype(np.uint8) * rng.integers(1, 255, size=(2, N, N), dtype=np.uint8)
    perm = rng.permutation(N).astype(np.int32)
    pt = torch.from_numpy(perm).cuda()
    out = bbm.bbm_permute_mask(torch.from_numpy(mask).cuda(), pt)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.permute_mask(mask, perm))
    for d in (64, 128):
        x = make_qkv(2, 3, N, d, seed=8)[0]
        xt = bf16_tensor(x)
        g = bbm.bbm_gather_rows(xt, pt)
        back = bbm.bbm_gather_rows(g, pt, inverse=True)
        torch.cuda.synchronize()
        assert np.array_equal(g.view(torch.int16).cpu().numpy().view(np.uint16), x[:, :, perm])
        assert torch.equal(back.view(torch.int16), xt.view(torch.int16))


def test_reordered_pipeline_equals_attention_on_the_original_problem():
    """Scrambled graph mask -> ordering, permuted mask, gathered Q/K/V, block index, attention, O scattered back: the
    result is the oracle's attention on the ORIGINAL mask, and the reordering cut the non-zero blocks."""
    bbm = _bbm()
    B, H, N, d = 1, 2, 2048, 64
    A = masks.graph_mask(N, 11, reorder="none", xm=10.0, cap=100)
    q, k, v = make_qkv(B, H, N, d, seed=12)
    O_ref, lse_ref = oracle.masked_attention(q, k, v, A)
    mt = torch.from_numpy(A).cuda()
    perm = bbm.bbm_rcm_order(mt[0])
    pm = bbm.bbm_permute_mask(mt, perm)
    qp, kp, vp = (bbm.bbm_gather_rows(bf16_tensor(x), perm) for x in (q, k, v))
    idx = bbm.build_index(pm, 128, 64)
    op, lsep = bbm.bbm_attn_fwd(qp, kp, vp, idx)
    o = bbm.bbm_gather_rows(op, perm, inverse=True)
    lse = torch.empty_like(lsep)
    lse[:, :, perm.long()] = lsep
    torch.cuda.synchronize()
    assert_attention_close(o, lse, O_ref, lse_ref)
    before = int((bbm.build_index(mt, 128, 64).blk_class != 0).sum())
    after = int((idx.blk_class != 0).sum())
    assert after < before // 2, (before, after)
    want = oracle.reverse_cuthill_mckee(A[0])
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), want)


def test_full_size_graph_workload_ordering_and_block_reduction():
    """The scrambled graph of the largest configuration (N = 32768, about 10 million edges): the ordering equals the
    oracle's, and it cuts the non-zero 128 x 64 blocks as the host-side reordering of the workload generator does."""
    bbm = _bbm()
    from workloads import make_config
    cfg = make_config("C5", with_qkv=False)
    A = masks.graph_mask(cfg["N"], cfg["seed"], reorder="none")
    mt = torch.from_numpy(A).cuda()
    print("rcm full size: gpu", flush=True)
    perm = bbm.bbm_rcm_order(mt[0])
    pm = bbm.bbm_permute_mask(mt, perm)
    torch.cuda.synchronize()
    print("rcm full size: oracle", flush=True)
    want = oracle.reverse_cuthill_mckee(A[0])
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), want)
    after = int((bbm.build_index(pm, 128, 64).blk_class != 0).sum())
    host = int((bbm.build_index(torch.from_numpy(cfg["mask"]).cuda(), 128, 64).blk_class != 0).sum())
    before = int((bbm.build_index(mt, 128, 64).blk_class != 0).sum())
    assert before == 256 * 512 and after <= host * 1.05 and after < before // 5, (before, after, host)
