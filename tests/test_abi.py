"""CPU-only checks of the boundary: the library loads, exports every declared symbol, and rejects bad
arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bbm():
    import paper_2409_15097_amd as m
    return m


def test_every_declared_symbol_is_exported(bbm):
    hdr = open(os.path.join(ROOT, "include", "bbm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(bbm_[a-z0-9_]+)\s*\(", hdr))
    assert names == {"bbm_last_error", "bbm_version", "bbm_build_block_mask", "bbm_build_runs",
                     "bbm_build_sparse_index", "bbm_build_index", "bbm_sched_bytes", "bbm_attn_fwd_workspace_bytes",
                     "bbm_attn_fwd", "bbm_build_col_index", "bbm_col_sched_bytes", "bbm_attn_bwd_workspace_bytes",
                     "bbm_attn_bwd", "bbm_build_block_mask_rect", "bbm_attn_fwd_rect", "bbm_rcm_workspace_bytes",
                     "bbm_rcm_order", "bbm_permute_mask", "bbm_gather_rows", "bbm_attn_fwd_static",
                     "bbm_probe_mfma_bf16", "bbm_probe_mfma_bf16_flop"}
    raw = C.CDLL(bbm.library_path())
    for n in names:
        assert getattr(raw, n) is not None
    assert bbm.bbm_version() >= 100


def test_binding_has_the_same_names(bbm):
    for n in ("bbm_last_error", "bbm_version", "bbm_build_block_mask", "bbm_build_runs", "bbm_build_sparse_index",
              "bbm_build_index",
              "bbm_sched_bytes", "bbm_attn_fwd_workspace_bytes", "bbm_attn_fwd", "bbm_build_col_index",
              "bbm_col_sched_bytes", "bbm_attn_bwd_workspace_bytes", "bbm_attn_bwd", "bbm_build_block_mask_rect",
              "bbm_attn_fwd_rect", "bbm_rcm_workspace_bytes", "bbm_rcm_order", "bbm_permute_mask", "bbm_gather_rows",
              "bbm_attn_fwd_static", "bbm_probe_mfma_bf16", "bbm_probe_mfma_bf16_flop"):
        assert callable(getattr(bbm, n))


FAKE = C.c_void_p(0x1000)      # never dereferenced: validation fails first


def test_build_block_mask_rejects_bad_arguments(bbm):
    L = bbm.lib
    assert L.bbm_build_block_mask(None, 1, 64, 64, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL
    assert "NULL" in bbm.bbm_last_error()
    assert L.bbm_build_block_mask(FAKE, 1, 64, 64, 64, 64, None, None, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_block_mask(FAKE, 0, 64, 64, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_block_mask(FAKE, 1, 0, 64, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_block_mask(FAKE, 1, 64, 63, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_block_mask(FAKE, 1, 64, 64, 0, 64, FAKE, None, None, None) == bbm.BBM_EUNSUPPORTED
    assert L.bbm_build_block_mask(FAKE, 1, 64, 64, 257, 64, FAKE, None, None, None) == bbm.BBM_EUNSUPPORTED
    assert L.bbm_build_block_mask(FAKE, 1, 64, 64, 64, 48, FAKE, None, None, None) == bbm.BBM_EUNSUPPORTED
    assert L.bbm_build_block_mask(FAKE, 1, 64, 64, 64, 64, FAKE, None, C.c_void_p(0x1004), None) == bbm.BBM_EINVAL


def test_index_builders_reject_bad_arguments(bbm):
    L = bbm.lib
    assert L.bbm_build_runs(None, 1, 4, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == bbm.BBM_EINVAL
    assert L.bbm_build_runs(FAKE, 1, 4, 4, FAKE, None, FAKE, FAKE, FAKE, None) == bbm.BBM_EINVAL
    assert L.bbm_build_runs(FAKE, 1, 0, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == bbm.BBM_EINVAL
    assert L.bbm_build_sparse_index(FAKE, 1, 4, 4, None, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_sparse_index(FAKE, 1, 4, 0, FAKE, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_sparse_index(FAKE, 1, 1 << 20, 1 << 20, FAKE, FAKE, None, None) == bbm.BBM_EUNSUPPORTED
    assert L.bbm_build_sparse_index(FAKE, 1, 4, 4, FAKE, FAKE, C.c_void_p(0x1004), None) == bbm.BBM_EINVAL
    # the one-call form reports the same errors as the two stages
    assert L.bbm_build_index(FAKE, 1, 4, 4, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_index(FAKE, 1, 4, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_index(FAKE, 1, 4, 4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, C.c_void_p(0x1004), None) == bbm.BBM_EINVAL
    assert L.bbm_build_index(FAKE, 1, 0, 4, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None) == bbm.BBM_EINVAL
    assert bbm.bbm_sched_bytes(1, 4) == 4 * (8 + 12 * 4) and bbm.bbm_sched_bytes(0, 4) == 0


def _idx(bbm, Br=128, Bc=64, Mb=1, N=256, **ptrs):
    from paper_2409_15097_amd.binding import _CIndex
    s = _CIndex(Br, Bc, Mb, -(-N // Br), -(-N // Bc), N, N, *([None] * 13))
    for k, v in ptrs.items():
        setattr(s, k, v)
    return s


def _attn(bbm, idx, q=FAKE, k=FAKE, v=FAKE, o=FAKE, B=1, H=1, N=256, d=64, scale=0.125, Mb=1, packed=FAKE, mode=None,
          ws_bytes=0):
    mode = bbm.BBM_MODE_DENSE_BASELINE if mode is None else mode
    return bbm.lib.bbm_attn_fwd(q, k, v, o, None, B, H, N, d, scale, Mb, packed, C.byref(idx) if idx else None, mode,
                                None, ws_bytes, None)


def test_attn_fwd_rejects_bad_arguments(bbm):
    idx = _idx(bbm)
    assert _attn(bbm, idx, q=None) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, o=C.c_void_p(0x1008)) == bbm.BBM_EINVAL and "aligned" in bbm.bbm_last_error()
    assert _attn(bbm, idx, B=0) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, scale=0.0) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, scale=float("nan")) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, scale=float("inf")) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, B=4, Mb=2) == bbm.BBM_EINVAL
    assert _attn(bbm, None) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, packed=None) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, d=96) == bbm.BBM_EUNSUPPORTED
    assert _attn(bbm, _idx(bbm, Bc=32)) == bbm.BBM_EUNSUPPORTED
    assert _attn(bbm, _idx(bbm, Br=32)) == bbm.BBM_EUNSUPPORTED
    assert _attn(bbm, _idx(bbm, N=512)) == bbm.BBM_EINVAL and "does not match" in bbm.bbm_last_error()
    assert _attn(bbm, idx, mode=17) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, mode=bbm.BBM_MODE_BITMAP) == bbm.BBM_EINVAL and "bin_blk_mat" in bbm.bbm_last_error()
    assert _attn(bbm, idx, mode=bbm.BBM_MODE_RUNS) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, mode=bbm.BBM_MODE_LIST) == bbm.BBM_EINVAL
    assert _attn(bbm, idx, mode=bbm.BBM_MODE_AUTO) == bbm.BBM_EINVAL          # AUTO falls back to BITMAP, which needs bin_blk_mat
    # the mask-everywhere baseline takes the zeros of empty blocks from the class bytes (their packed words are not written)
    assert _attn(bbm, idx, mode=bbm.BBM_MODE_DENSE_BASELINE) == bbm.BBM_EINVAL and "blk_class" in bbm.bbm_last_error()


def test_index_built_for_another_length_is_refused_even_with_equal_block_counts(bbm):
    """N = 200 and N = 256 both give 2 x 4 blocks at 128 x 64, but the packed mask's row stride differs."""
    idx = _idx(bbm, N=200)
    assert (idx.nbr, idx.nbc) == (2, 4)
    assert _attn(bbm, idx, N=256) == bbm.BBM_EINVAL and "does not match" in bbm.bbm_last_error()
    assert _bwd(bbm, _idx(bbm, N=200, row_ptr=0x2000, col_idx=0x3000, col_ptr=0x4000, row_idx=0x5000), N=256) == bbm.BBM_EINVAL
    assert "does not match" in bbm.bbm_last_error()


def test_static_scratch_entry_point_validates_like_the_workspace_one_and_states_its_limit(bbm):
    L = bbm.lib
    idx = _idx(bbm, row_ptr=0x2000, col_idx=0x3000, sched=0x4000)
    call = lambda B=1, H=1, N=256, q=FAKE, index=idx, mode=bbm.BBM_MODE_LIST: L.bbm_attn_fwd_static(
        q, FAKE, FAKE, FAKE, None, B, H, N, N, 64, 0.125, 1, FAKE, C.byref(index), mode, None)
    assert call(q=None) == bbm.BBM_EINVAL and "bbm_attn_fwd_static" in bbm.bbm_last_error()
    assert call(N=512) == bbm.BBM_EINVAL
    assert call(mode=17) == bbm.BBM_EINVAL
    assert call(index=_idx(bbm), mode=bbm.BBM_MODE_LIST) == bbm.BBM_EINVAL       # LIST needs the list
    # 2^23 block rows x heads: 32 MiB of counters alone do not fit the static scratch
    big = _idx(bbm, N=65536, Br=64, row_ptr=0x2000, col_idx=0x3000, sched=0x4000)
    assert call(B=64, H=128, N=65536, index=big) == bbm.BBM_EWORKSPACE
    assert "static scratch" in bbm.bbm_last_error() and "bbm_attn_fwd_rect" in bbm.bbm_last_error()


def test_workspace_query_and_check(bbm):
    need = bbm.bbm_attn_fwd_workspace_bytes(4, 16, 4096, 64, 128, 64, bbm.BBM_MODE_LIST)
    assert need > 0 and need == bbm.bbm_attn_fwd_workspace_bytes(4, 16, 4096, 64, 128, 64, bbm.BBM_MODE_AUTO)
    assert bbm.bbm_attn_fwd_workspace_bytes(4, 16, 4096, 64, 128, 64, bbm.BBM_MODE_BITMAP) == 0
    assert bbm.bbm_attn_fwd_workspace_bytes(0, 16, 4096, 64, 128, 64, bbm.BBM_MODE_LIST) == 0
    # counters (8 + B*H*nbr ints, rounded to 256 bytes) + partial records of (d/2 + 2) * 2*Br floats, capped at 32 MiB
    assert need == 8448 + (32 << 20)
    assert bbm.bbm_attn_fwd_workspace_bytes(4, 8, 2048, 64, 128, 64, bbm.BBM_MODE_LIST) == 2304 + 512 * 34 * 256 * 4
    # B*H*nbr = 256 work-groups: still a small launch if its rows are long, 2 parts per block row
    assert bbm.bbm_attn_fwd_workspace_bytes(2, 8, 2048, 64, 128, 64, bbm.BBM_MODE_LIST) == 1280 + 256 * 2 * 34 * 256 * 4
    # a small launch (B*H*nbr = 64 work-groups): 8 parts per block row, each parking a record
    assert bbm.bbm_attn_fwd_workspace_bytes(1, 32, 256, 128, 128, 64, bbm.BBM_MODE_LIST) == 512 + 64 * 8 * 66 * 256 * 4
    # BITMAP and RUNS ask for the same on a small launch (optional there) and for nothing otherwise
    for mode in (bbm.BBM_MODE_BITMAP, bbm.BBM_MODE_RUNS):
        assert bbm.bbm_attn_fwd_workspace_bytes(1, 32, 256, 128, 128, 64, mode) == 512 + 64 * 8 * 66 * 256 * 4
        assert bbm.bbm_attn_fwd_workspace_bytes(2, 8, 2048, 64, 128, 64, mode) == 1280 + 256 * 2 * 34 * 256 * 4
        assert bbm.bbm_attn_fwd_workspace_bytes(4, 8, 2048, 64, 128, 64, mode) == 0
    assert bbm.bbm_attn_fwd_workspace_bytes(1, 32, 256, 128, 128, 64, bbm.BBM_MODE_DENSE_BASELINE) == 0
    idx = _idx(bbm, row_ptr=0x2000, col_idx=0x3000, sched=0x4000)
    assert _attn(bbm, idx, mode=bbm.BBM_MODE_LIST) == bbm.BBM_EWORKSPACE          # no workspace given
    assert "workspace" in bbm.bbm_last_error()


def _bwd(bbm, idx, q=FAKE, do=FAKE, lse=FAKE, dk=FAKE, B=1, H=1, N=256, d=64, scale=0.125, Mb=1, packed=FAKE, ws=FAKE,
         ws_bytes=1 << 30):
    return bbm.lib.bbm_attn_bwd(q, FAKE, FAKE, FAKE, do, lse, FAKE, dk, FAKE, B, H, N, d, scale, Mb, packed,
                                C.byref(idx) if idx else None, ws, ws_bytes, None)


def test_attn_bwd_and_col_index_reject_bad_arguments(bbm):
    L = bbm.lib
    assert L.bbm_build_col_index(None, 1, 4, 4, FAKE, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_col_index(FAKE, 1, 4, 4, None, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_col_index(FAKE, 1, 4, 0, FAKE, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_col_index(FAKE, 1, 1 << 20, 1 << 20, FAKE, FAKE, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_col_index(FAKE, 1, 4, 4, FAKE, FAKE, C.c_void_p(0x1004), None) == bbm.BBM_EINVAL
    assert bbm.bbm_col_sched_bytes(2, 5) == 4 * (8 + 12 * 10) and bbm.bbm_col_sched_bytes(0, 5) == 0
    need = bbm.bbm_attn_bwd_workspace_bytes(2, 3, 100, 64, 128)
    assert need >= 2 * 4 * 600 + 3 * 4 * 600 * 64 and bbm.bbm_attn_bwd_workspace_bytes(0, 3, 100, 64, 128) == 0
    assert bbm.bbm_attn_bwd_workspace_bytes(2, 3, 100, 96, 128) == 0 and bbm.bbm_attn_bwd_workspace_bytes(2, 3, 100, 64, 32) == 0
    full = _idx(bbm, row_ptr=0x2000, col_idx=0x3000, col_ptr=0x4000, row_idx=0x5000)
    assert _bwd(bbm, full, q=None) == bbm.BBM_EINVAL
    assert _bwd(bbm, full, lse=None) == bbm.BBM_EINVAL
    assert _bwd(bbm, full, dk=C.c_void_p(0x1008)) == bbm.BBM_EINVAL and "aligned" in bbm.bbm_last_error()
    assert _bwd(bbm, full, scale=0.0) == bbm.BBM_EINVAL
    assert _bwd(bbm, full, B=4, Mb=2) == bbm.BBM_EINVAL
    assert _bwd(bbm, None) == bbm.BBM_EINVAL
    assert _bwd(bbm, full, packed=None) == bbm.BBM_EINVAL
    assert _bwd(bbm, full, d=96) == bbm.BBM_EUNSUPPORTED
    assert _bwd(bbm, _idx(bbm, Br=32, row_ptr=0x2000, col_idx=0x3000, col_ptr=0x4000, row_idx=0x5000)) == bbm.BBM_EUNSUPPORTED
    assert _bwd(bbm, _idx(bbm, N=512, row_ptr=0x2000, col_idx=0x3000, col_ptr=0x4000, row_idx=0x5000)) == bbm.BBM_EINVAL
    assert _bwd(bbm, _idx(bbm, row_ptr=0x2000, col_idx=0x3000)) == bbm.BBM_EINVAL and "column list" in bbm.bbm_last_error()
    assert _bwd(bbm, full, ws=None) == bbm.BBM_EWORKSPACE
    assert _bwd(bbm, full, ws_bytes=16) == bbm.BBM_EWORKSPACE
    assert _bwd(bbm, full, ws=C.c_void_p(0x1008)) == bbm.BBM_EINVAL


def test_rectangular_entry_points_reject_bad_arguments(bbm):
    L = bbm.lib
    assert L.bbm_build_block_mask_rect(None, 1, 64, 128, 128, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_block_mask_rect(FAKE, 1, 64, 0, 128, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL
    assert L.bbm_build_block_mask_rect(FAKE, 1, 64, 128, 127, 64, 64, FAKE, None, None, None) == bbm.BBM_EINVAL   # stride < columns
    assert "bbm_build_block_mask_rect" in bbm.bbm_last_error()
    idx = _idx(bbm, N=256)                                     # nbr = 2, nbc = 4: fits Nq = 256, Nk = 256 only
    rect = lambda Nq, Nk, **kw: L.bbm_attn_fwd_rect(kw.get("q", FAKE), FAKE, FAKE, FAKE, None, 1, 1, Nq, Nk, 64, 0.125, 1, FAKE,
                                                    C.byref(idx), bbm.BBM_MODE_DENSE_BASELINE, None, 0, None)
    assert rect(256, 0) == bbm.BBM_EINVAL
    assert rect(256, 512) == bbm.BBM_EINVAL and "does not match" in bbm.bbm_last_error()
    assert rect(512, 256) == bbm.BBM_EINVAL
    assert rect(256, 256, q=None) == bbm.BBM_EINVAL and "bbm_attn_fwd_rect" in bbm.bbm_last_error()


def test_reorder_entry_points_reject_bad_arguments(bbm):
    L = bbm.lib
    need = bbm.bbm_rcm_workspace_bytes(1000)
    assert need >= 1000 * 16 * 8 + 24 * 1000 and bbm.bbm_rcm_workspace_bytes(0) == 0 and bbm.bbm_rcm_workspace_bytes(70000) == 0
    assert L.bbm_rcm_order(None, 64, 64, FAKE, FAKE, 1 << 30, None) == bbm.BBM_EINVAL
    assert L.bbm_rcm_order(FAKE, 64, 63, FAKE, FAKE, 1 << 30, None) == bbm.BBM_EINVAL
    assert L.bbm_rcm_order(FAKE, 70000, 70000, FAKE, FAKE, 1 << 40, None) == bbm.BBM_EUNSUPPORTED
    assert L.bbm_rcm_order(FAKE, 64, 64, FAKE, FAKE, 16, None) == bbm.BBM_EWORKSPACE
    assert L.bbm_rcm_order(FAKE, 64, 64, FAKE, None, 0, None) == bbm.BBM_EWORKSPACE
    assert L.bbm_permute_mask(FAKE, 1, 64, 64, None, C.c_void_p(0x2000), None) == bbm.BBM_EINVAL
    assert L.bbm_permute_mask(FAKE, 1, 64, 64, FAKE, FAKE, None) == bbm.BBM_EINVAL and "input" in bbm.bbm_last_error()
    assert L.bbm_permute_mask(FAKE, 1, 70000, 70000, FAKE, C.c_void_p(0x2000), None) == bbm.BBM_EUNSUPPORTED
    assert L.bbm_gather_rows(FAKE, FAKE, C.c_void_p(0x2000), 2, 64, 60, 0, None) == bbm.BBM_EINVAL
    assert L.bbm_gather_rows(FAKE, FAKE, C.c_void_p(0x2008), 2, 64, 64, 0, None) == bbm.BBM_EINVAL
    assert L.bbm_gather_rows(FAKE, FAKE, FAKE, 2, 64, 64, 0, None) == bbm.BBM_EINVAL


def test_matrix_probe_validates_and_counts_its_flop(bbm):
    L = bbm.lib
    assert L.bbm_probe_mfma_bf16(1, 1000, None, None) == bbm.BBM_EINVAL and "sink" in bbm.bbm_last_error()
    assert L.bbm_probe_mfma_bf16(1, 0, FAKE, None) == bbm.BBM_EINVAL
    assert L.bbm_probe_mfma_bf16(0, (1 << 24) + 1, FAKE, None) == bbm.BBM_EINVAL
    # 256 work-groups x 4 waves x 16 instructions x 32*32*16 multiply-adds
    assert bbm.bbm_probe_mfma_bf16_flop(1000) == 256 * 4 * 16 * 1000 * 2 * 32 * 32 * 16
    assert bbm.bbm_probe_mfma_bf16_flop(0) == 0.0


def test_package_imports_without_the_library_and_fails_loudly_at_first_use():
    """`python -m paper_2409_15097_amd.build` has to import the package before a library exists; every use of the
    binding without one raises (there is no fallback)."""
    import subprocess, sys
    code = ("import paper_2409_15097_amd as bbm\n"
            "try:\n    bbm.bbm_version()\nexcept ImportError as e:\n    print('IMPORT-ERROR', 'no fallback' in str(e))\n"
            "else:\n    print('LOADED')\n")
    env = dict(os.environ, BBM_LIBRARY="/nonexistent/libbbm.so")
    out = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert out.stdout.strip() == "IMPORT-ERROR True", out.stdout + out.stderr
