"""GPU parity: backward pass of the fused masked attention (dQ, dK, dV) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from workloads import masks, make_qkv, small_variant, make_config
from gpu_util import bf16_tensor, bf16_result_to_f64, assert_grad_close, assert_index_equal, index_to_numpy

pytestmark = pytest.mark.gpu


def _bbm():
    import paper_2409_15097_amd as bbm
    return bbm


def _d_o(B, H, N, d, seed=991):
    return make_qkv(B, H, N, d, seed=seed)[0]          # upstream gradient: seeded bf16 N(0,1), like the inputs


def _gpu_grads(cfg, do_bits, Br, scale=None, idx=None):
    bbm = _bbm()
    if idx is None:
        idx = bbm.build_index(torch.from_numpy(cfg["mask"]).cuda(), Br, 64, columns=True)
    q, k, v = (bf16_tensor(cfg[x]) for x in "qkv")
    o, lse = bbm.bbm_attn_fwd(q, k, v, idx, softmax_scale=scale)
    dq, dk, dv = bbm.bbm_attn_bwd(q, k, v, o, bf16_tensor(do_bits), lse, idx, softmax_scale=scale)
    torch.cuda.synchronize()
    return dq, dk, dv


def _check(grads, ref, mags, tag=None):
    for name, g, r, m in zip(("dQ", "dK", "dV"), grads, ref, mags):
        assert_grad_close(name, bf16_result_to_f64(g), r, mag=m, tag=tag)


@pytest.mark.parametrize("Br", [64, 128, 256])
@pytest.mark.parametrize("N", [200, 1000, 77])
def test_column_index_matches_oracle(N, Br):
    bbm = _bbm()
    mask = np.stack([masks.random_blocks(64 * (-(-N // 64)), N + s, blk=32, p_empty=0.5, p_full=0.3)[0][:N, :N] for s in (1, 2)])
    idx = bbm.build_index(torch.from_numpy(np.ascontiguousarray(mask)).cuda(), Br, 64, columns=True)
    torch.cuda.synchronize()
    assert_index_equal(index_to_numpy(idx), mask, Br, 64)


def test_column_index_of_a_plane_with_more_than_4096_block_columns():
    """The class matrix is given directly (a mask with that many block columns would not fit): columns are not sorted
    by length then but listed from the last to the first."""
    bbm = _bbm()
    from paper_2409_15097_amd.binding import BlockIndex
    rng = np.random.default_rng(41)
    cls = rng.integers(0, 3, size=(2, 3, 4100)).astype(np.uint8)
    cls[:, :, 7] = 0
    idx = BlockIndex(128, 64, 2, 3, 4100, 4100 * 64, blk_class=torch.from_numpy(cls).cuda())
    bbm.bbm_build_col_index(idx)
    torch.cuda.synchronize()
    cp, ri = oracle.column_index(cls)
    cs = oracle.column_schedule(cp, ri)
    assert np.array_equal(idx.col_ptr.cpu().numpy(), cp)
    got_ri = idx.row_idx.cpu().numpy().view(np.uint32)
    for m in range(2):
        assert np.array_equal(got_ri[m * 12300: m * 12300 + cp[m, -1]], ri[m * 12300: m * 12300 + cp[m, -1]])
    got = idx.col_sched.cpu().numpy()
    n = 8 + 8 * int(cs[0])
    assert np.array_equal(got[:n], cs[:n]) and np.array_equal(got[-4 * 2 * 4100:], cs[-4 * 2 * 4100:])
    assert got[-4 * 4100:].reshape(4100, 4)[:, 0].tolist() == list(range(4099, -1, -1))


def test_column_index_of_planes_with_more_than_64_block_rows():
    """Class matrices of more than 64 block rows take the three-launch path (one wave per block column, 64 block rows
    per ballot step): 130 rows = two full steps and a ragged one, 71 columns = a ragged last work-group, an empty and a
    completely full column, two planes."""
    bbm = _bbm()
    from paper_2409_15097_amd.binding import BlockIndex
    rng = np.random.default_rng(43)
    Mb, nbr, nbc = 2, 130, 71
    cls = rng.choice(np.array([0, 0, 1, 2], dtype=np.uint8), size=(Mb, nbr, nbc))
    cls[:, :, 5] = 0
    cls[1, :, 9] = 2
    idx = BlockIndex(128, 64, Mb, nbr, nbc, nbc * 64, blk_class=torch.from_numpy(cls).cuda())
    bbm.bbm_build_col_index(idx)
    torch.cuda.synchronize()
    cp, ri = oracle.column_index(cls)
    cs = oracle.column_schedule(cp, ri)
    assert np.array_equal(idx.col_ptr.cpu().numpy(), cp)
    got_ri = idx.row_idx.cpu().numpy().view(np.uint32)
    cap = nbr * nbc
    for m in range(Mb):
        assert np.array_equal(got_ri[m * cap: m * cap + cp[m, -1]], ri[m * cap: m * cap + cp[m, -1]])
    assert np.array_equal(idx.col_sched.cpu().numpy(), cs)


SMALL = [("C1", 256, 1, 2), ("C2", 1024, 2, 2), ("C3", 640, 1, 2), ("C4", 2048, 1, 2), ("C5", 2048, 1, 2),
         ("C0d", 512, 1, 2), ("C0c", 512, 1, 2), ("C2b", 1024, 2, 2), ("C4w", 1024, 1, 2), ("C4d", 1024, 1, 2)]


@pytest.mark.parametrize("name,N,B,H", SMALL)
def test_small_variants(name, N, B, H):
    cfg = small_variant(name, N=N, B=B, H=H)
    do = _d_o(*cfg["q"].shape)
    ref = oracle.masked_attention_bwd(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do)
    mags = oracle.masked_attention_bwd_magnitudes(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do)
    first = None
    bbm = _bbm()
    for Br in (64, 128, 256):
        print(f"bwd case {name} N={N} Br={Br}", flush=True)
        idx = bbm.build_index(torch.from_numpy(cfg["mask"]).cuda(), Br, 64, columns=True)
        grads = _gpu_grads(cfg, do, Br, idx=idx)
        _check(grads, ref, mags, tag=f"bwd small {name} N={N} Br={Br}")
        # one lane owns one query (dQ) resp. one key (dK, dV) and walks its tiles in ascending order whatever the
        # block height; blocks that are skipped or unmasked at one height and not at another contribute exact zeros.
        # So, unless a schedule cut a row or column into parts (another order of the sums), the bits do not depend on Br
        if int(idx.sched[0]) == 0 and int(idx.col_sched[0]) == 0:
            bits = [g.view(torch.int16) for g in grads]
            if first is None:
                first = bits
            else:
                assert all(torch.equal(a, b) for a, b in zip(bits, first))


@pytest.mark.parametrize("N", [200, 333, 77, 1, 65, 1000])
@pytest.mark.parametrize("d", [64, 128])
def test_ragged_sizes_with_empty_rows_and_unattended_keys(N, d):
    B, H = 2, 3
    q, k, v = make_qkv(B, H, N, d, seed=N + d)
    do = _d_o(B, H, N, d, seed=N + d + 5)
    rng = np.random.default_rng(N)
    m = masks.random_blocks(64 * (-(-N // 64)), N + 1, blk=32, p_empty=0.4, p_full=0.3)[0][:N, :N].copy()
    empty = rng.integers(0, N, size=max(1, N // 10))
    m[empty] = 0                                             # fully masked query rows
    dead = rng.integers(0, N, size=max(1, N // 10))
    mask = np.stack([m, np.roll(m, 3, axis=1)])
    mask[:, :, dead] = 0                                     # keys nobody attends
    cfg = dict(q=q, k=k, v=v, mask=mask)
    ref = oracle.masked_attention_bwd(q, k, v, mask, do)
    mags = oracle.masked_attention_bwd_magnitudes(q, k, v, mask, do)
    for Br in (64, 128, 256):
        print(f"bwd ragged N={N} d={d} Br={Br}", flush=True)
        dq, dk, dv = _gpu_grads(cfg, do, Br)
        _check((dq, dk, dv), ref, mags, tag=f"bwd ragged N={N} d={d} Br={Br}")
        assert torch.all(dq[0, :, empty] == 0)
        assert torch.all(dk[:, :, dead] == 0) and torch.all(dv[:, :, dead] == 0)


def test_custom_scale_d128():
    """Scales flatter and sharper than 1/sqrt(d) against the same bars."""
    cfg = small_variant("C3", N=640, B=2, H=2)
    do = _d_o(*cfg["q"].shape)
    for scale in (0.05, 0.3):
        ref = oracle.masked_attention_bwd(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do, scale=scale)
        mags = oracle.masked_attention_bwd_magnitudes(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do, scale=scale)
        _check(_gpu_grads(cfg, do, 128, scale=scale), ref, mags, tag=f"bwd C3 N=640 scale={scale}")


def test_single_allowed_key_routes_dO_to_dV():
    """One allowed key per query: P = 1 exactly, so dS = 0 and dV_j is the sum of the dO rows that chose key j."""
    B, H, N, d = 1, 2, 320, 64
    q, k, v = make_qkv(B, H, N, d, seed=3)
    do = _d_o(B, H, N, d)
    pi = np.random.default_rng(3).permutation(N)
    mask = np.zeros((1, N, N), dtype=np.uint8)
    mask[0, np.arange(N), pi] = 1
    dq, dk, dv = _gpu_grads(dict(q=q, k=k, v=v, mask=mask), do, 64)
    want = np.zeros((B, H, N, d))
    want[:, :, pi] = oracle.bf16_bits_to_f64(do)
    # the stored lse carries the rounding of Q*scale*log2(e): P = exp(s' - lse) is 1 up to that, not bit-exactly
    assert np.abs(bf16_result_to_f64(dv) - want).max() <= 2e-2 * np.abs(want).max()
    assert np.abs(bf16_result_to_f64(dq)).max() <= 2e-2 and np.abs(bf16_result_to_f64(dk)).max() <= 2e-2


@pytest.mark.parametrize("d", [64, 128])
def test_key_permutation_permutes_dk_dv_and_leaves_dq(d):
    """Permuting keys/values together with the mask columns scrambles the block matrix (and with it every list,
    schedule and skipped tile); dQ must not move and dK, dV must move with their keys."""
    cfg = small_variant("C2", N=1024, B=1, H=2)
    if d == 128:
        q, k, v = make_qkv(1, 2, 1024, 128, seed=77)
        cfg = dict(cfg, q=q, k=k, v=v)
    do = _d_o(*cfg["q"].shape)
    pi = np.random.default_rng(5).permutation(1024)
    cfg2 = dict(q=cfg["q"], k=cfg["k"][:, :, pi].copy(), v=cfg["v"][:, :, pi].copy(), mask=cfg["mask"][:, :, pi].copy())
    dq2, dk2, dv2 = (bf16_result_to_f64(g) for g in _gpu_grads(cfg2, do, 128))
    ref = oracle.masked_attention_bwd(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do)
    mags = oracle.masked_attention_bwd_magnitudes(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do)
    assert_grad_close("dQ", dq2, ref[0], mag=mags[0], tag=f"bwd key permutation d={d}")
    assert_grad_close("dK", dk2, ref[1][:, :, pi], mag=mags[1][:, :, pi], tag=f"bwd key permutation d={d}")
    assert_grad_close("dV", dv2, ref[2][:, :, pi], mag=mags[2][:, :, pi], tag=f"bwd key permutation d={d}")


def test_deterministic():
    cfg = small_variant("C4", N=2048, B=1, H=2)
    do = _d_o(*cfg["q"].shape)
    a = _gpu_grads(cfg, do, 128)
    b = _gpu_grads(cfg, do, 128)
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


# Full-size parity in bench.py's launch configuration: "all" = every element of dQ, dK, dV; otherwise whole (batch, head)
# slices (all query rows and all keys of the head, so cut block rows and cut block columns are in) plus sampled query
# rows (dQ) and sampled keys (dK, dV) in the other heads.
FULL_SIZE = {"C2": "all", "C2b": "all", "C3": "all", "C4": [(0, 0), (0, 15)], "C4w": [(0, 5)], "C4d": [(0, 9)],
             "C5": [(0, 0)]}


@pytest.mark.parametrize("name", list(FULL_SIZE))
def test_full_size_whole_gradients(name):
    bbm = _bbm()
    cfg = make_config(name)
    B, H, N, d = cfg["B"], cfg["H"], cfg["N"], cfg["d"]
    do = _d_o(B, H, N, d)
    whole = FULL_SIZE[name]
    heads = [(b, h) for b in range(B) for h in range(H)] if whole == "all" else whole
    print(f"bwd full {name}: oracle on {len(heads)} whole (batch, head) slices", flush=True)
    if whole == "all":
        ref = oracle.masked_attention_bwd(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do)
        mags = oracle.masked_attention_bwd_magnitudes(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do)
    else:
        ref = [np.zeros((len(heads), N, d)) for _ in range(3)]
        mags = [np.zeros((len(heads), N, d)) for _ in range(3)]
        for n, (b, h) in enumerate(heads):
            mb = cfg["mask"][b:b + 1] if cfg["mask"].shape[0] == B else cfg["mask"]
            args = (cfg["q"][b:b + 1, h:h + 1], cfg["k"][b:b + 1, h:h + 1], cfg["v"][b:b + 1, h:h + 1], mb, do[b:b + 1, h:h + 1])
            for r, g in zip(ref, oracle.masked_attention_bwd(*args)):
                r[n] = g[0, 0]
            for r, g in zip(mags, oracle.masked_attention_bwd_magnitudes(*args)):
                r[n] = g[0, 0]
        rng = np.random.default_rng(17)
        others = [(b, h) for b in range(B) for h in range(H) if (b, h) not in heads]
        rows = sorted((*others[int(rng.integers(len(others)))], int(rng.integers(N))) for _ in range(96)) + [(B - 1, H - 1, N - 1)]
        cols = sorted((*others[int(rng.integers(len(others)))], int(rng.integers(N))) for _ in range(24)) + [(B - 1, H - 1, 0)]
        dq_ref = oracle.masked_attention_bwd_rows(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do, rows)
        dk_ref, dv_ref = oracle.masked_attention_bwd_cols(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], do, cols)
    print(f"bwd full {name}: gpu", flush=True)
    dq, dk, dv = _gpu_grads(cfg, do, 128)
    for g in (dq, dk, dv):
        assert not torch.isnan(g.float()).any()
    tag = f"bwd {name} Br=128"
    if whole == "all":
        _check((dq, dk, dv), ref, mags, tag=tag)
    else:
        bi, hi = (torch.tensor(x, device="cuda") for x in zip(*heads))
        _check((dq[bi, hi], dk[bi, hi], dv[bi, hi]), ref, mags, tag=tag)
        bi, hi, ri = (torch.tensor(x, device="cuda") for x in zip(*rows))
        assert_grad_close("dQ", bf16_result_to_f64(dq[bi, hi, ri]), dq_ref, tag=tag + " sampled")
        bi, hi, ci = (torch.tensor(x, device="cuda") for x in zip(*cols))
        assert_grad_close("dK", bf16_result_to_f64(dk[bi, hi, ci]), dk_ref, tag=tag + " sampled")
        assert_grad_close("dV", bf16_result_to_f64(dv[bi, hi, ci]), dv_ref, tag=tag + " sampled")
    empty = np.flatnonzero(cfg["mask"][0].sum(axis=1) == 0)
    if empty.size:
        assert torch.all(dq[0, :, torch.from_numpy(empty).cuda()] == 0)


def test_lists_longer_than_one_window():
    """A block row and a block column with more entries than one LDS list window (256): global query rows that see
    every key, global keys that every query sees, a band elsewhere; ragged N."""
    B, H, N, d, Br = 1, 1, 16500, 64, 64
    q, k, v = make_qkv(B, H, N, d, seed=31)
    do = _d_o(B, H, N, d, seed=32)
    i = np.arange(N)
    mask = (np.abs(i[:, None] - i[None, :]) <= 40).astype(np.uint8)
    mask[:, :64] = 1
    mask[100:132] = 1
    cfg = dict(q=q, k=k, v=v, mask=mask[None])
    bbm = _bbm()
    idx = bbm.build_index(torch.from_numpy(cfg["mask"]).cuda(), Br, 64, columns=True)
    rp, cp = idx.row_ptr.cpu().numpy()[0], idx.col_ptr.cpu().numpy()[0]
    assert (rp[1:] - rp[:-1]).max() == 258 and (cp[1:] - cp[:-1]).max() == 258
    rows = [(0, 0, r) for r in (0, 100, 131, 132, 5000, 16447, 16448, 16499)]
    cols = [(0, 0, c) for c in (0, 63, 64, 120, 9000, 16499)]
    dq_ref = oracle.masked_attention_bwd_rows(q, k, v, cfg["mask"], do, rows)
    dk_ref, dv_ref = oracle.masked_attention_bwd_cols(q, k, v, cfg["mask"], do, cols)
    dq, dk, dv = _gpu_grads(cfg, do, Br, idx=idx)
    assert_grad_close("dQ", bf16_result_to_f64(dq[0, 0, [r for _, _, r in rows]]), dq_ref)
    assert_grad_close("dK", bf16_result_to_f64(dk[0, 0, [c for _, _, c in cols]]), dk_ref)
    assert_grad_close("dV", bf16_result_to_f64(dv[0, 0, [c for _, _, c in cols]]), dv_ref)
    for g in (dq, dk, dv):
        assert not torch.isnan(g.float()).any()


@pytest.mark.parametrize("Br", [64, 128, 256])
def test_cut_rows_and_columns_with_a_mask_shared_by_the_batch(Br):
    """A few block rows and block columns far longer than the rest: the split schedules cut them into parts that
    several work-groups compute and one adds up; the mask is shared by B = 3 batch entries.  The same zero-filled
    workspace serves two calls in a row and must be back to zeros (its counters) afterwards."""
    B, H, N, d = 3, 2, 4096, 64
    q, k, v = make_qkv(B, H, N, d, seed=21)
    do = _d_o(B, H, N, d, seed=22)
    i = np.arange(N)
    m = (np.abs(i[:, None] - i[None, :]) <= 70).astype(np.uint8)
    m[300:340] = 1                                   # "global" query rows that see every key
    m[:, 1000:1030] = 1                              # "global" keys that every query sees
    m[2000:2003, ::3] = 1                            # a sparse long row: every tile partial
    m[3900:3910] = 0                                 # fully masked rows
    cfg = dict(q=q, k=k, v=v, mask=m[None])
    bbm = _bbm()
    idx = bbm.build_index(torch.from_numpy(cfg["mask"]).cuda(), Br, 64, columns=True)
    assert_index_equal(index_to_numpy(idx), cfg["mask"], Br, 64)
    assert idx.sched.cpu().numpy()[0] >= 4 and (Br == 256 or idx.col_sched.cpu().numpy()[0] >= 2)   # 16 block rows at Br = 256: no column is long
    ref = oracle.masked_attention_bwd(q, k, v, cfg["mask"], do)
    mags = oracle.masked_attention_bwd_magnitudes(q, k, v, cfg["mask"], do)
    qt, kt, vt, dot = (bf16_tensor(x) for x in (q, k, v, do))
    o, lse = bbm.bbm_attn_fwd(qt, kt, vt, idx)
    ws = torch.zeros(bbm.bbm_attn_bwd_workspace_bytes(B, H, N, d, Br), dtype=torch.uint8, device="cuda")
    g1 = bbm.bbm_attn_bwd(qt, kt, vt, o, dot, lse, idx, workspace=ws)
    g1 = [g.clone() for g in g1]
    g2 = bbm.bbm_attn_bwd(qt, kt, vt, o, dot, lse, idx, workspace=ws)
    torch.cuda.synchronize()
    _check(g1, ref, mags, tag=f"bwd cut rows and columns Br={Br}")
    for a, b in zip(g1, g2):                         # parts are summed in part order: the same bits on every run
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    nbr, nbc = idx.nbr, idx.nbc
    counters = ws[:4 * (8 + B * H * nbr) + 4 * (8 + B * H * nbc) + 512].view(torch.int32)
    assert int(counters[:8 + B * H * nbr].abs().sum()) == 0
    # without the schedules (no cut): the same values up to the order of the sums
    idx.sched, idx.col_sched = None, None
    g3 = bbm.bbm_attn_bwd(qt, kt, vt, o, dot, lse, idx)
    torch.cuda.synchronize()
    _check(g3, ref, mags)
