"""GPU parity: fused masked attention forward against the fp64 oracle (O within 2e-2 max-abs / 2e-3 mean-abs)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import masks, make_qkv, small_variant, make_config
from gpu_util import bf16_tensor, bf16_result_to_f64, assert_attention_close, O_MAX_ABS, O_MEAN_ABS, LSE_MAX_ABS

pytestmark = pytest.mark.gpu


def _bbm():
    import paper_2409_15097_amd as bbm
    return bbm


MODES = ["BITMAP", "RUNS", "LIST", "DENSE_BASELINE", "AUTO"]


def _mode(bbm, name):
    return getattr(bbm, "BBM_MODE_" + name)


def _gpu_attn(cfg, Br, mode, scale=None):
    bbm = _bbm()
    mask = torch.from_numpy(cfg["mask"]).cuda()
    idx = bbm.build_index(mask, Br, 64)
    q, k, v = (bf16_tensor(cfg[x]) for x in "qkv")
    o, lse = bbm.bbm_attn_fwd(q, k, v, idx, mode=_mode(bbm, mode), softmax_scale=scale)
    torch.cuda.synchronize()
    return o, lse


SMALL = [("C1", 256, 1, 2), ("C2", 1024, 2, 2), ("C3", 640, 1, 2), ("C4", 2048, 1, 2), ("C5", 2048, 1, 2),
         ("C0d", 512, 1, 2), ("C0c", 512, 1, 2), ("C2b", 1024, 2, 2), ("C4w", 1024, 1, 2), ("C4d", 1024, 1, 2)]


@pytest.mark.parametrize("name,N,B,H", SMALL)
@pytest.mark.parametrize("Br", [64, 128, 256])
def test_small_variants_all_modes(name, N, B, H, Br):
    cfg = small_variant(name, N=N, B=B, H=H)
    O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"])
    outs = {}
    for mode in MODES:
        print(f"case {name} N={N} Br={Br} mode={mode}", flush=True)
        o, lse = _gpu_attn(cfg, Br, mode)
        assert_attention_close(o, lse, O_ref, lse_ref)
        outs[mode] = (o, lse)
    # same tile visit order and same arithmetic in the schedules that walk a whole block row in one work-group
    assert torch.equal(outs["RUNS"][0].view(torch.int16), outs["BITMAP"][0].view(torch.int16))
    # AUTO is LIST; LIST may cut long rows into parts, which only changes the rounding order
    assert torch.equal(outs["AUTO"][0].view(torch.int16), outs["LIST"][0].view(torch.int16))
    assert torch.equal(outs["AUTO"][1], outs["LIST"][1])


@pytest.mark.parametrize("N", [200, 333, 77, 1, 65, 1000])
@pytest.mark.parametrize("d", [64, 128])
def test_ragged_sizes_with_empty_rows(N, d):
    B, H = 2, 3
    q, k, v = make_qkv(B, H, N, d, seed=N + d)
    rng = np.random.default_rng(N)
    m = masks.random_blocks(64 * (-(-N // 64)), N + 1, blk=32, p_empty=0.4, p_full=0.3)[0][:N, :N].copy()
    m[rng.integers(0, N, size=max(1, N // 10))] = 0        # fully masked rows
    cfg = dict(q=q, k=k, v=v, mask=np.stack([m, np.roll(m, 3, axis=1)]))
    O_ref, lse_ref = oracle.masked_attention(q, k, v, cfg["mask"])
    for Br in (64, 128, 256):
        for mode in MODES:
            print(f"ragged N={N} d={d} Br={Br} mode={mode}", flush=True)
            o, lse = _gpu_attn(cfg, Br, mode)
            assert_attention_close(o, lse, O_ref, lse_ref)
            rows = np.flatnonzero(~np.isfinite(lse_ref[0, 0]))
            assert torch.all(o[0, :, rows] == 0)


@pytest.mark.parametrize("name,N", [("C3", 640), ("C2", 1024)])
def test_custom_scales_meet_the_same_bars(name, N):
    """Softmax scales flatter and sharper than 1/sqrt(d), at d = 128 (tree) and d = 64 (packed): the same bars at every
    scale.  (Scales above 1/sqrt(d) run the kernel instances that keep the non-power-of-two part of the scale out of
    the bf16 operand.)"""
    cfg = small_variant(name, N=N, B=2, H=2)
    d = cfg["q"].shape[-1]
    for scale in (None, 0.05, d ** -0.5 * 1.01, 0.3, 0.5):
        O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], scale=scale)
        for mode in MODES:
            o, lse = _gpu_attn(cfg, 128, mode, scale=scale)
            assert_attention_close(o, lse, O_ref, lse_ref, tag=f"fwd {name} N={N} scale={scale} {mode}")


@pytest.mark.parametrize("Br", [64, 128, 256])
def test_index_rebuilt_in_place_for_a_sparser_mask(Br):
    """The block reduction writes packed words only for (block row x 64 column) slabs that hold a set bit, so an index
    rebuilt in place keeps the previous mask's words wherever the new mask has an empty block.  No schedule may see
    them, the mask-everywhere baseline included."""
    from gpu_util import index_to_numpy, assert_index_equal
    bbm = _bbm()
    cfg = small_variant("C4", N=1024, B=1, H=2)
    O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"])
    q, k, v = (bf16_tensor(cfg[x]) for x in "qkv")
    idx = bbm.build_index(torch.ones((1, 1024, 1024), dtype=torch.uint8, device="cuda"), Br, 64)
    assert bool((idx.packed_mask == -1).all())                       # the all-ones mask: every word written, all bits set
    mask = torch.from_numpy(cfg["mask"]).cuda()
    bbm.build_index(mask, Br, 64, idx=idx)
    torch.cuda.synchronize()
    assert_index_equal(index_to_numpy(idx), cfg["mask"], Br, 64)
    cls = idx.blk_class.cpu().numpy()[0]
    assert (cls == 0).any()
    words = idx.packed_mask.cpu().numpy()[0]                             # [W][N]
    for i, j in np.argwhere(cls == 0)[:50]:
        assert np.all(words[j, i * Br:(i + 1) * Br] == -1)           # untouched: still the old mask's words
    for mode in MODES:
        print(f"rebuilt index Br={Br} mode={mode}", flush=True)
        o, lse = bbm.bbm_attn_fwd(q, k, v, idx, mode=_mode(bbm, mode))
        torch.cuda.synchronize()
        assert_attention_close(o, lse, O_ref, lse_ref)


def test_key_permutation_changes_blocks_but_not_output():
    """Permuting keys/values together with the mask columns scrambles the block matrix; O must not move."""
    cfg = small_variant("C2", N=1024, B=1, H=2)
    pi = np.random.default_rng(0).permutation(1024)
    cfg2 = dict(q=cfg["q"], k=cfg["k"][:, :, pi].copy(), v=cfg["v"][:, :, pi].copy(), mask=cfg["mask"][:, :, pi].copy())
    o1, _ = _gpu_attn(cfg, 128, "LIST")
    o2, _ = _gpu_attn(cfg2, 128, "LIST")
    a, b = bf16_result_to_f64(o1), bf16_result_to_f64(o2)
    assert np.abs(a - b).max() <= O_MAX_ABS
    O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"])
    assert np.abs(b - O_ref).max() <= O_MAX_ABS and np.abs(b - O_ref).mean() <= O_MEAN_ABS


def test_single_allowed_key_returns_value_bits_exactly():
    B, H, N, d = 1, 2, 320, 64
    q, k, v = make_qkv(B, H, N, d, seed=3)
    pi = np.random.default_rng(3).permutation(N)
    mask = np.zeros((1, N, N), dtype=np.uint8)
    mask[0, np.arange(N), pi] = 1
    o, lse = _gpu_attn(dict(q=q, k=k, v=v, mask=mask), 64, "LIST")
    got = o.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, v[:, :, pi])
    _, lse_ref = oracle.masked_attention(q, k, v, mask)
    assert np.abs(lse.cpu().numpy() - lse_ref).max() <= LSE_MAX_ABS


def test_deterministic():
    cfg = small_variant("C4", N=2048, B=1, H=2)
    o1, l1 = _gpu_attn(cfg, 128, "LIST")
    o2, l2 = _gpu_attn(cfg, 128, "LIST")
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)


@pytest.mark.parametrize("name", ["C3q", "C3qL"])
def test_full_size_decode_shapes(name):
    """The two decode-time bench rows (tree tokens as the only queries; C3qL is the small launch that computes every
    block row in parts) at their full sizes and in bench.py's configuration, every output against the oracle."""
    bbm = _bbm()
    cfg = make_config(name)
    assert cfg["q"].shape[2] != cfg["k"].shape[2]
    O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"])
    for Br, mode in ((128, "AUTO"), (64, "LIST"), (128, "BITMAP")):
        print(f"full {name} Br={Br} mode={mode}", flush=True)
        o, lse = _gpu_attn_rect(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], Br, mode)
        assert_attention_close(o, lse, O_ref, lse_ref)


# Full-size parity, in bench.py's launch configuration.  "all": the oracle evaluates the whole output.  Otherwise a
# list of (batch, head) slices that are compared whole -- every block row of the head, so the rows the schedule cut
# (global tokens), the first and the last block row are all in -- plus sampled rows in the other heads.
FULL_SIZE = {"C2": "all", "C2b": "all", "C3": "all", "C4": [(0, 0), (0, 15)], "C4w": [(0, 5)], "C4d": [(0, 9)],
             "C5": [(0, 0)]}


@pytest.mark.parametrize("name", list(FULL_SIZE))
def test_full_size_whole_outputs(name):
    bbm = _bbm()
    cfg = make_config(name)
    B, H, N, d = cfg["B"], cfg["H"], cfg["N"], cfg["d"]
    whole = FULL_SIZE[name]
    heads = [(b, h) for b in range(B) for h in range(H)] if whole == "all" else whole
    print(f"full {name}: oracle on {len(heads)} whole (batch, head) slices", flush=True)
    if whole == "all":
        O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"])
    else:
        O_ref = np.zeros((len(heads), N, d))
        lse_ref = np.zeros((len(heads), N))
        for n, (b, h) in enumerate(heads):
            mb = cfg["mask"][b:b + 1] if cfg["mask"].shape[0] == B else cfg["mask"]
            o1, l1 = oracle.masked_attention(cfg["q"][b:b + 1, h:h + 1], cfg["k"][b:b + 1, h:h + 1], cfg["v"][b:b + 1, h:h + 1], mb)
            O_ref[n], lse_ref[n] = o1[0, 0], l1[0, 0]
    # sampled rows in the heads that are not compared whole
    rng = np.random.default_rng(7)
    rows = []
    if whole != "all":
        others = [(b, h) for b in range(B) for h in range(H) if (b, h) not in heads]
        rows = sorted((*others[int(rng.integers(len(others)))], int(rng.integers(N))) for _ in range(192))
        rows += [(B - 1, H - 1, N - 1), (B - 1, H - 1, 0)]
        Or_ref, lr_ref = oracle.masked_attention_rows(cfg["q"], cfg["k"], cfg["v"], cfg["mask"], rows)
    empty = np.flatnonzero(cfg["mask"][0].sum(axis=1) == 0)
    mask = torch.from_numpy(cfg["mask"]).cuda()
    q, k, v = (bf16_tensor(cfg[x]) for x in "qkv")
    ref_bits = None
    for Br, mode in ((128, "AUTO"), (128, "RUNS"), (128, "BITMAP"), (64, "LIST")):
        print(f"full {name} Br={Br} mode={mode}", flush=True)
        idx = bbm.build_index(mask, Br, 64)
        o, lse = bbm.bbm_attn_fwd(q, k, v, idx, mode=_mode(bbm, mode))
        torch.cuda.synchronize()
        assert not torch.isnan(o.float()).any()
        tag = f"fwd {name} Br={Br} {mode}"
        if whole == "all":
            assert_attention_close(o, lse, O_ref, lse_ref, tag=tag)
        else:
            bi, hi = (torch.tensor(x, device="cuda") for x in zip(*heads))
            assert_attention_close(o[bi, hi], lse[bi, hi], O_ref, lse_ref, tag=tag)      # mean-abs over whole heads
            bi, hi, ri = (torch.tensor(x, device="cuda") for x in zip(*rows))
            assert_attention_close(o[bi, hi, ri], lse[bi, hi, ri], Or_ref, lr_ref, tag=tag + " sampled rows")
        if Br == 128 and mode in ("RUNS", "BITMAP"):
            bits = o.view(torch.int16)
            if ref_bits is None:
                ref_bits = bits.clone()
            else:
                assert torch.equal(bits, ref_bits)
        # properties that hold at any size: fully masked rows are exactly zero
        if empty.size:
            assert torch.all(o[0, :, torch.from_numpy(empty).cuda()] == 0)


def test_tile_lists_longer_than_one_window():
    """nbc = 1025 block columns: every schedule needs a second window of its LDS tile list (window = 1024 entries).
    All-ones mask built on the device; the oracle evaluates sampled rows (plain softmax rows here)."""
    bbm = _bbm()
    N, d, Br = 65600, 64, 128                       # 1025 x 64 columns; 512.5 x 128 rows: the last block row is ragged
    q, k, v = make_qkv(1, 1, N, d, seed=11)
    mask = torch.ones((1, N, N), dtype=torch.uint8, device="cuda")
    idx = bbm.build_index(mask, Br, 64)
    torch.cuda.synchronize()
    nbr, nbc = idx.nbr, idx.nbc
    assert (nbr, nbc) == (513, 1025)
    cls = idx.blk_class.cpu().numpy()
    assert np.all(cls[0, :-1] == 2) and np.all(cls[0, -1] == 1)           # the ragged block row holds padding: partial
    assert np.array_equal(idx.row_ptr.cpu().numpy()[0], 1025 * np.arange(nbr + 1))
    ci = idx.col_idx.cpu().numpy().view(np.uint32)[:nbr * nbc].reshape(nbr, nbc)
    assert np.array_equal(ci[:-1], np.broadcast_to(np.arange(nbc, dtype=np.uint32) | np.uint32(1 << 31), (nbr - 1, nbc)))
    assert np.array_equal(ci[-1], np.arange(nbc, dtype=np.uint32))
    sched = idx.sched.cpu().numpy()
    assert sched[0] == 0 and sched[1] == 2050                             # nothing cut: rows are walked window by window
    rows = [(0, 0, r) for r in (0, 1, 127, 128, 4097, 33000, 65471, 65472, 65535, 65536, 65599)]
    ones_rows = np.broadcast_to(np.ones((1, 1, N), dtype=np.uint8), (1, N, N))
    O_ref, lse_ref = oracle.masked_attention_rows(q, k, v, ones_rows, rows)
    qt, kt, vt = (bf16_tensor(x) for x in (q, k, v))
    ri = torch.tensor([r for _, _, r in rows], device="cuda")
    for mode in ("LIST", "RUNS", "BITMAP"):
        print(f"two-window lists, mode={mode}", flush=True)
        o, lse = bbm.bbm_attn_fwd(qt, kt, vt, idx, mode=_mode(bbm, mode))
        torch.cuda.synchronize()
        err = np.abs(bf16_result_to_f64(o[0, 0, ri]) - O_ref)
        assert err.max() <= O_MAX_ABS and err.mean() <= O_MEAN_ABS
        assert np.abs(lse[0, 0, ri].cpu().numpy().astype(np.float64) - lse_ref).max() <= LSE_MAX_ABS
        assert not torch.isnan(o.float()).any()


@pytest.mark.parametrize("Br", [64, 128, 256])
def test_cut_rows_with_a_mask_shared_by_the_batch(Br):
    """A few block rows with 64 tiles among rows with 3: the split schedule cuts them into parts that several
    work-groups compute and one merges; the mask is shared by B = 3 batch entries (parts x (batch, head) items)."""
    B, H, N, d = 3, 2, 4096, 64
    q, k, v = make_qkv(B, H, N, d, seed=21)
    i = np.arange(N)
    m = (np.abs(i[:, None] - i[None, :]) <= 70).astype(np.uint8)
    m[300:340] = 1                                   # "global" query rows that see every key
    m[2000:2003, ::3] = 1                            # and a sparse long row: every tile partial
    m[3900:3910] = 0                                 # fully masked rows
    cfg = dict(q=q, k=k, v=v, mask=m[None])
    bbm = _bbm()
    idx = bbm.build_index(torch.from_numpy(cfg["mask"]).cuda(), Br, 64)
    sched = idx.sched.cpu().numpy()
    assert sched[0] >= 4 and sched[2] >= 2           # parts exist, from at least two cut rows
    O_ref, lse_ref = oracle.masked_attention(q, k, v, cfg["mask"])
    for mode in ("LIST", "AUTO", "BITMAP"):
        o, lse = _gpu_attn(cfg, Br, mode)
        assert_attention_close(o, lse, O_ref, lse_ref)
    o1, l1 = _gpu_attn(cfg, Br, "LIST")              # merging in part order: the same bits on every run
    o2, l2 = _gpu_attn(cfg, Br, "LIST")
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)


def _gpu_attn_rect(q, k, v, mask, Br, mode, check_index=False):
    bbm = _bbm()
    idx = bbm.build_index(torch.from_numpy(np.ascontiguousarray(mask)).cuda(), Br, 64)
    if check_index:
        from gpu_util import assert_index_equal, index_to_numpy
        assert_index_equal(index_to_numpy(idx), mask, Br, 64)
    o, lse = bbm.bbm_attn_fwd_rect(bf16_tensor(q), bf16_tensor(k), bf16_tensor(v), idx, mode=_mode(bbm, mode))
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("Br", [64, 128, 256])
def test_tree_verification_at_decode_time_new_queries_against_the_cache(Br):
    """Nq != Nk: the 200 candidate-tree tokens are the only queries; keys are the 1024-token prefix plus the tree
    (the rows of the square tree-verification mask that belong to the tree)."""
    B, H, d, prefix, tree = 2, 2, 128, 1024, 200
    full = masks.tree_verification(prefix, masks.random_subtree([10, 5, 3, 2], tree, 77))      # [1, 1224, 1224]
    mask = np.ascontiguousarray(full[:, prefix:])                                              # [1, 200, 1224]
    q = make_qkv(B, H, tree, d, seed=5)[0]
    _, k, v = make_qkv(B, H, prefix + tree, d, seed=6)
    O_ref, lse_ref = oracle.masked_attention(q, k, v, mask)
    for mode in MODES:
        print(f"decode-time tree Br={Br} mode={mode}", flush=True)
        o, lse = _gpu_attn_rect(q, k, v, mask, Br, mode, check_index=(mode == "LIST"))
        assert o.shape == (B, H, tree, d) and lse.shape == (B, H, tree)
        assert_attention_close(o, lse, O_ref, lse_ref)


@pytest.mark.parametrize("Nq,Nk", [(1, 65), (77, 1000), (300, 130), (129, 64), (64, 4097)])
@pytest.mark.parametrize("d", [64, 128])
def test_rectangular_ragged_sizes_with_empty_rows(Nq, Nk, d):
    B, H = 2, 2
    q = make_qkv(B, H, Nq, d, seed=Nq + d)[0]
    _, k, v = make_qkv(B, H, Nk, d, seed=Nk + d)
    side = 64 * (-(-max(Nq, Nk) // 64))
    m = masks.random_blocks(side, Nq + Nk, blk=32, p_empty=0.4, p_full=0.3)[0][:Nq, :Nk].copy()
    m[np.random.default_rng(Nq).integers(0, Nq, size=max(1, Nq // 10))] = 0
    mask = np.stack([m, np.roll(m, 5, axis=1)])
    O_ref, lse_ref = oracle.masked_attention(q, k, v, mask)
    for Br in (64, 128, 256):
        for mode in MODES:
            print(f"rect Nq={Nq} Nk={Nk} d={d} Br={Br} mode={mode}", flush=True)
            o, lse = _gpu_attn_rect(q, k, v, mask, Br, mode, check_index=(mode == "BITMAP"))
            assert_attention_close(o, lse, O_ref, lse_ref)


def test_small_launch_computes_every_block_row_in_parts():
    """Fewer than 256 work-groups (one sequence, a few block rows of new tokens against a long cache): LIST mode
    computes every block row in parts.  Rows with fewer tiles than parts, empty rows, a workspace reused by two calls
    (bit-identical results, counters back to zero), and agreement with the one-work-group-per-row schedules."""
    bbm = _bbm()
    B, H, d, Nq, Nk = 1, 3, 64, 300, 16400          # 257 block columns: 8 parts per block row
    q = make_qkv(B, H, Nq, d, seed=41)[0]
    _, k, v = make_qkv(B, H, Nk, d, seed=42)
    rng = np.random.default_rng(43)
    mask = (rng.random((1, Nq, Nk)) < 0.3).astype(np.uint8)
    mask[0, :, 3000:9000] = 1                      # full tiles, too
    mask[0, :70, 200:] = 0                         # a block row with 4 tiles only (fewer than the 8 parts)
    mask[0, 128:192] = 0                           # an empty block row at Br = 64
    mask[0, 250:260, :] = 1
    O_ref, lse_ref = oracle.masked_attention(q, k, v, mask)
    for Br in (64, 128, 256):
        idx = bbm.build_index(torch.from_numpy(mask).cuda(), Br, 64)
        need = bbm.bbm_attn_fwd_workspace_bytes(B, H, Nq, d, Br, 64, bbm.BBM_MODE_LIST)
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
        qt, kt, vt = (bf16_tensor(x) for x in (q, k, v))
        o1, l1 = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=bbm.BBM_MODE_LIST, workspace=ws)
        o1, l1 = o1.clone(), l1.clone()
        o2, l2 = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=bbm.BBM_MODE_LIST, workspace=ws)
        torch.cuda.synchronize()
        assert_attention_close(o1, l1, O_ref, lse_ref)
        assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)
        nbr = idx.nbr
        assert int(ws[:4 * (8 + B * H * nbr)].view(torch.int32).abs().sum()) == 0
        # BITMAP and RUNS compute the block rows of a small launch in parts, too (equal shares of the block columns), when
        # they get the workspace; with none to speak of they run one work-group per block row: same values up to the
        # rounding order of the merge, and the workspace comes back with its counters at zero
        none = torch.zeros(16, dtype=torch.uint8, device="cuda")
        for mode in (bbm.BBM_MODE_BITMAP, bbm.BBM_MODE_RUNS):
            os_, ls_ = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=mode, workspace=ws)
            os_, ls_ = os_.clone(), ls_.clone()
            ou, lu = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=mode, workspace=none)
            torch.cuda.synchronize()
            assert_attention_close(os_, ls_, O_ref, lse_ref)
            assert_attention_close(ou, lu, O_ref, lse_ref)
            assert not torch.equal(os_.view(torch.int16), ou.view(torch.int16))          # really another order of the sums
            assert np.abs(bf16_result_to_f64(os_) - bf16_result_to_f64(ou)).max() <= O_MAX_ABS
            assert int(ws[:4 * (8 + B * H * nbr)].view(torch.int32).abs().sum()) == 0
            assert torch.all(os_[0, :, 128:192] == 0)
        assert torch.all(o1[0, :, 128:192] == 0)


@pytest.mark.parametrize("d", [64, 128])
def test_launch_of_128_to_256_work_groups_over_long_rows_is_computed_in_parts(d):
    """One sequence, 8 heads, 2048 new queries against 8300 keys (130 block columns): 256 work-groups at Br = 64 and 128
    at Br = 128 (2 parts each: at least 64 block columns per part), 64 at Br = 256 (4 parts of at least 32).  Every
    schedule against the oracle, and against its own unsplit run."""
    bbm = _bbm()
    B, H, Nq, Nk = 1, 8, 2048, 8300
    q = make_qkv(B, H, Nq, d, seed=51)[0]
    _, k, v = make_qkv(B, H, Nk, d, seed=52)
    rng = np.random.default_rng(53)
    i, j = np.arange(Nq)[:, None], np.arange(Nk)[None, :]
    mask = (j <= i + (Nk - Nq)).astype(np.uint8)[None]          # causal, aligned to the end of the cache
    mask[0] &= (rng.random((Nq, Nk)) < 0.9).astype(np.uint8)     # with holes: partial tiles everywhere
    mask[0, :, 1024:3072] = 1                                    # and a stretch of full ones
    mask[0, 700:830] = 0                                         # fully masked rows (a whole block row at Br = 64 and 128)
    O_ref, lse_ref = oracle.masked_attention(q, k, v, mask)
    qt, kt, vt = (bf16_tensor(x) for x in (q, k, v))
    none = torch.zeros(16, dtype=torch.uint8, device="cuda")
    for Br in (64, 128, 256):
        idx = bbm.build_index(torch.from_numpy(mask).cuda(), Br, 64)
        need = bbm.bbm_attn_fwd_workspace_bytes(B, H, Nq, d, Br, 64, bbm.BBM_MODE_BITMAP)
        parts = {64: 2, 128: 4, 256: 8}[Br]          # the query does not know the key count: room for 512 / work-groups parts
        assert need == -(-(8 + H * idx.nbr) * 4 // 256) * 256 + H * idx.nbr * parts * (d // 2 + 2) * 2 * Br * 4
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
        for mode in ("LIST", "BITMAP", "RUNS"):
            print(f"mid-size launch d={d} Br={Br} mode={mode}", flush=True)
            o, lse = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=_mode(bbm, mode), workspace=ws)
            torch.cuda.synchronize()
            assert_attention_close(o, lse, O_ref, lse_ref)
            assert int(ws[:4 * (8 + H * idx.nbr)].view(torch.int32).abs().sum()) == 0
            if mode != "LIST":                                   # LIST cannot run without its workspace
                ou, lu = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=_mode(bbm, mode), workspace=none)
                torch.cuda.synchronize()
                assert_attention_close(ou, lu, O_ref, lse_ref)
                assert not torch.equal(o.view(torch.int16), ou.view(torch.int16))      # another order of the sums
