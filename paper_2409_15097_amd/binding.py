"""ctypes binding of libbbm.so.  Argument marshalling only; see include/bbm.h for the contract."""
import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

BBM_OK, BBM_EINVAL, BBM_EUNSUPPORTED, BBM_EWORKSPACE, BBM_EHIP = 0, -1, -2, -3, -4
BBM_MODE_BITMAP, BBM_MODE_RUNS, BBM_MODE_LIST, BBM_MODE_DENSE_BASELINE, BBM_MODE_AUTO = 0, 1, 2, 3, 4

# BBM_LIBRARY names another build of the same library (the host-sanitizer build of the argument checks, say)
_LIB_PATH = os.environ.get("BBM_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbbm.so")


class BbmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libbbm error {code}: {msg}")
        self.code = code


class _CIndex(C.Structure):
    _fields_ = [("Br", C.c_int32), ("Bc", C.c_int32), ("Mb", C.c_int64), ("nbr", C.c_int64), ("nbc", C.c_int64),
                ("Nq", C.c_int64), ("Nk", C.c_int64),
                ("blk_class", C.c_void_p), ("bin_blk_mat", C.c_void_p), ("offset", C.c_void_p),
                ("total_ones", C.c_void_p), ("nz_lo", C.c_void_p), ("nz_hi", C.c_void_p), ("nz_cnt", C.c_void_p),
                ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("sched", C.c_void_p),
                ("col_ptr", C.c_void_p), ("row_idx", C.c_void_p), ("col_sched", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it first (python -m paper_2409_15097_amd.build); "
                          "there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    i64, vp, ci = C.c_int64, C.c_void_p, C.c_int
    L.bbm_last_error.restype = C.c_char_p
    L.bbm_last_error.argtypes = []
    L.bbm_version.restype = ci
    L.bbm_version.argtypes = []
    L.bbm_build_block_mask.restype = ci
    L.bbm_build_block_mask.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp, vp, vp]
    L.bbm_build_block_mask_rect.restype = ci
    L.bbm_build_block_mask_rect.argtypes = [vp, i64, i64, i64, i64, ci, ci, vp, vp, vp, vp]
    L.bbm_attn_fwd_rect.restype = ci
    L.bbm_attn_fwd_rect.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, C.c_float, i64, vp, C.POINTER(_CIndex), ci,
                                    vp, C.c_size_t, vp]
    L.bbm_attn_fwd_static.restype = ci
    L.bbm_attn_fwd_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, C.c_float, i64, vp, C.POINTER(_CIndex), ci, vp]
    L.bbm_build_runs.restype = ci
    L.bbm_build_runs.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp]
    L.bbm_build_sparse_index.restype = ci
    L.bbm_build_sparse_index.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
    L.bbm_build_index.restype = ci
    L.bbm_build_index.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.bbm_sched_bytes.restype = C.c_size_t
    L.bbm_sched_bytes.argtypes = [i64, i64]
    L.bbm_attn_fwd_workspace_bytes.restype = C.c_size_t
    L.bbm_attn_fwd_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci, ci]
    L.bbm_attn_fwd.restype = ci
    L.bbm_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, C.c_float, i64, vp, C.POINTER(_CIndex), ci,
                               vp, C.c_size_t, vp]
    L.bbm_build_col_index.restype = ci
    L.bbm_build_col_index.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
    L.bbm_col_sched_bytes.restype = C.c_size_t
    L.bbm_col_sched_bytes.argtypes = [i64, i64]
    L.bbm_attn_bwd_workspace_bytes.restype = C.c_size_t
    L.bbm_attn_bwd_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    L.bbm_attn_bwd.restype = ci
    L.bbm_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, C.c_float, i64, vp,
                               C.POINTER(_CIndex), vp, C.c_size_t, vp]
    L.bbm_rcm_workspace_bytes.restype = C.c_size_t
    L.bbm_rcm_workspace_bytes.argtypes = [i64]
    L.bbm_rcm_order.restype = ci
    L.bbm_rcm_order.argtypes = [vp, i64, i64, vp, vp, C.c_size_t, vp]
    L.bbm_permute_mask.restype = ci
    L.bbm_permute_mask.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    L.bbm_gather_rows.restype = ci
    L.bbm_gather_rows.argtypes = [vp, vp, vp, i64, i64, ci, ci, vp]
    L.bbm_probe_mfma_bf16.restype = ci
    L.bbm_probe_mfma_bf16.argtypes = [ci, i64, vp, vp]
    L.bbm_probe_mfma_bf16_flop.restype = C.c_double
    L.bbm_probe_mfma_bf16_flop.argtypes = [i64]
    return L


lib = _load()


def bbm_last_error() -> str:
    return lib.bbm_last_error().decode()


def bbm_version() -> int:
    return lib.bbm_version()


def _check(rc: int):
    if rc != BBM_OK:
        raise BbmError(rc, bbm_last_error())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _cdiv(a, b):
    return -(-a // b)


@dataclass
class BlockIndex:
    """Device tensors of one preprocessed mask (all optional except the tile size and extents)."""
    Br: int
    Bc: int
    Mb: int
    nbr: int
    nbc: int
    N: int                      # query rows of the mask
    Nk: Optional[int] = None    # key columns (None: square, = N)
    blk_class: Optional[torch.Tensor] = None
    bin_blk_mat: Optional[torch.Tensor] = None
    packed_mask: Optional[torch.Tensor] = None
    offset: Optional[torch.Tensor] = None
    total_ones: Optional[torch.Tensor] = None
    nz_lo: Optional[torch.Tensor] = None
    nz_hi: Optional[torch.Tensor] = None
    nz_cnt: Optional[torch.Tensor] = None
    row_ptr: Optional[torch.Tensor] = None
    col_idx: Optional[torch.Tensor] = None
    sched: Optional[torch.Tensor] = None
    col_ptr: Optional[torch.Tensor] = None
    row_idx: Optional[torch.Tensor] = None
    col_sched: Optional[torch.Tensor] = None

    def c_struct(self) -> _CIndex:
        g = lambda t: None if t is None else t.data_ptr()
        return _CIndex(self.Br, self.Bc, self.Mb, self.nbr, self.nbc, self.N, self.N if self.Nk is None else self.Nk,
                       g(self.blk_class), g(self.bin_blk_mat),
                       g(self.offset), g(self.total_ones), g(self.nz_lo), g(self.nz_hi), g(self.nz_cnt),
                       g(self.row_ptr), g(self.col_idx), g(self.sched), g(self.col_ptr), g(self.row_idx), g(self.col_sched))


def bbm_build_block_mask(mask: torch.Tensor, Br: int, Bc: int, idx: Optional[BlockIndex] = None,
                         want_bin: bool = True, want_packed: bool = True, stream=None) -> BlockIndex:
    """mask: uint8 CUDA tensor [Mb,N,N] (row stride may exceed N).  Writes class / BinBlkMat / packed bits into
    idx's tensors (allocated here when idx is None) and returns idx."""
    assert mask.shape[1] == mask.shape[2]
    return bbm_build_block_mask_rect(mask, Br, Bc, idx=idx, want_bin=want_bin, want_packed=want_packed, stream=stream)


def bbm_build_block_mask_rect(mask: torch.Tensor, Br: int, Bc: int, idx: Optional[BlockIndex] = None,
                              want_bin: bool = True, want_packed: bool = True, stream=None) -> BlockIndex:
    """mask: uint8 CUDA tensor [Mb,Nq,Nk] (row stride may exceed Nk).  As bbm_build_block_mask; a square mask goes
    through the square entry point of the library."""
    assert mask.is_cuda and mask.dtype == torch.uint8 and mask.dim() == 3 and mask.stride(2) == 1
    Mb, N, Nk = mask.shape
    assert Mb == 1 or mask.stride(0) == N * mask.stride(1)
    nbr, nbc = _cdiv(N, Br), _cdiv(Nk, Bc)
    if idx is None:
        dev = mask.device
        idx = BlockIndex(Br, Bc, Mb, nbr, nbc, N, Nk=None if Nk == N else Nk)
        idx.blk_class = torch.empty((Mb, nbr, nbc), dtype=torch.uint8, device=dev)
        if want_bin:
            idx.bin_blk_mat = torch.empty((Mb, nbr, nbc), dtype=torch.uint8, device=dev)
        if want_packed:
            idx.packed_mask = torch.empty((Mb, _cdiv(Nk, 64), N), dtype=torch.int64, device=dev)
    if Nk == N:
        _check(lib.bbm_build_block_mask(_ptr(mask), Mb, N, mask.stride(1), Br, Bc, _ptr(idx.blk_class),
                                        _ptr(idx.bin_blk_mat), _ptr(idx.packed_mask), _stream(stream)))
    else:
        _check(lib.bbm_build_block_mask_rect(_ptr(mask), Mb, N, Nk, mask.stride(1), Br, Bc, _ptr(idx.blk_class),
                                             _ptr(idx.bin_blk_mat), _ptr(idx.packed_mask), _stream(stream)))
    return idx


def _alloc_runs(idx: BlockIndex):
    for name in ("offset", "total_ones", "nz_lo", "nz_hi", "nz_cnt"):
        if getattr(idx, name) is None:
            setattr(idx, name, torch.empty((idx.Mb, idx.nbr), dtype=torch.int32, device=idx.blk_class.device))


def _alloc_list(idx: BlockIndex):
    dev = idx.blk_class.device
    if idx.row_ptr is None:
        idx.row_ptr = torch.empty((idx.Mb, idx.nbr + 1), dtype=torch.int32, device=dev)
    if idx.col_idx is None:
        idx.col_idx = torch.zeros(idx.Mb * idx.nbr * idx.nbc, dtype=torch.int32, device=dev)
    if idx.sched is None:
        idx.sched = torch.empty(bbm_sched_bytes(idx.Mb, idx.nbr) // 4, dtype=torch.int32, device=dev)


def bbm_build_runs(idx: BlockIndex, stream=None) -> BlockIndex:
    _alloc_runs(idx)
    _check(lib.bbm_build_runs(_ptr(idx.blk_class), idx.Mb, idx.nbr, idx.nbc, _ptr(idx.offset), _ptr(idx.total_ones),
                              _ptr(idx.nz_lo), _ptr(idx.nz_hi), _ptr(idx.nz_cnt), _stream(stream)))
    return idx


def bbm_sched_bytes(Mb: int, nbr: int) -> int:
    return int(lib.bbm_sched_bytes(Mb, nbr))


def bbm_build_sparse_index(idx: BlockIndex, stream=None) -> BlockIndex:
    _alloc_list(idx)
    _check(lib.bbm_build_sparse_index(_ptr(idx.blk_class), idx.Mb, idx.nbr, idx.nbc, _ptr(idx.row_ptr),
                                      _ptr(idx.col_idx), _ptr(idx.sched), _stream(stream)))
    return idx


def bbm_build_index(idx: BlockIndex, stream=None) -> BlockIndex:
    """Run index, block list and schedule from idx.blk_class in one library call."""
    _alloc_runs(idx)
    _alloc_list(idx)
    _check(lib.bbm_build_index(_ptr(idx.blk_class), idx.Mb, idx.nbr, idx.nbc, _ptr(idx.offset), _ptr(idx.total_ones),
                               _ptr(idx.nz_lo), _ptr(idx.nz_hi), _ptr(idx.nz_cnt), _ptr(idx.row_ptr), _ptr(idx.col_idx),
                               _ptr(idx.sched), _stream(stream)))
    return idx


def bbm_build_col_index(idx: BlockIndex, stream=None) -> BlockIndex:
    """Per-column block list (what the backward pass walks for dK and dV) from idx.blk_class."""
    dev = idx.blk_class.device
    if idx.col_ptr is None:
        idx.col_ptr = torch.empty((idx.Mb, idx.nbc + 1), dtype=torch.int32, device=dev)
    if idx.row_idx is None:
        idx.row_idx = torch.zeros(idx.Mb * idx.nbr * idx.nbc, dtype=torch.int32, device=dev)
    if idx.col_sched is None:
        idx.col_sched = torch.empty(bbm_col_sched_bytes(idx.Mb, idx.nbc) // 4, dtype=torch.int32, device=dev)
    _check(lib.bbm_build_col_index(_ptr(idx.blk_class), idx.Mb, idx.nbr, idx.nbc, _ptr(idx.col_ptr), _ptr(idx.row_idx),
                                   _ptr(idx.col_sched), _stream(stream)))
    return idx


def bbm_col_sched_bytes(Mb: int, nbc: int) -> int:
    return int(lib.bbm_col_sched_bytes(Mb, nbc))


def build_index(mask: torch.Tensor, Br: int, Bc: int = 64, idx: Optional[BlockIndex] = None, stream=None,
                fused: bool = True, columns: bool = False) -> BlockIndex:
    """The whole preprocessing stage: block classes, then run index + block list + schedule (through the one-call
    entry point, or with fused=False through the two separate ones); columns=True adds the per-column list the
    backward pass needs."""
    idx = bbm_build_block_mask_rect(mask, Br, Bc, idx=idx, stream=stream)
    if fused:
        bbm_build_index(idx, stream=stream)
    else:
        bbm_build_runs(idx, stream=stream)
        bbm_build_sparse_index(idx, stream=stream)
    if columns:
        bbm_build_col_index(idx, stream=stream)
    return idx


def bf16_from_bits(bits) -> torch.Tensor:
    """numpy uint16 array of bf16 bit patterns -> bf16 CUDA tensor with the identical bits."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bbm_attn_fwd_workspace_bytes(B, H, N, d, Br, Bc, mode) -> int:
    return int(lib.bbm_attn_fwd_workspace_bytes(B, H, N, d, Br, Bc, mode))


def bbm_attn_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx: BlockIndex, mode: int = BBM_MODE_AUTO,
                 softmax_scale: Optional[float] = None, out: Optional[torch.Tensor] = None,
                 lse: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """q, k, v: bf16 CUDA tensors [B,H,N,d], contiguous.  Returns (O bf16 [B,H,N,d], lse fp32 [B,H,N])."""
    assert k.shape == q.shape
    return bbm_attn_fwd_rect(q, k, v, idx, mode=mode, softmax_scale=softmax_scale, out=out, lse=lse, workspace=workspace,
                             stream=stream)


_workspaces = {}


def _cached_workspace(kind: str, nbytes: int, device, stream, shape) -> torch.Tensor:
    """One workspace per (kind, device, stream), grown on demand.  The library leaves its counters at zero after every
    call, but where the counters end and the partial results begin depends on the problem's shape: the workspace is
    zero-filled when it is allocated and again whenever the shape changes (on the stream that uses it)."""
    key = (kind, device.index, _stream(stream).value)
    ws, last_shape = _workspaces.get(key, (None, None))
    if ws is None or ws.numel() < nbytes:
        ws = torch.zeros(max(16, nbytes), dtype=torch.uint8, device=device)
        torch.cuda.synchronize(device)          # zero before any stream may use it
    elif last_shape != shape:
        with (torch.cuda.stream(stream) if stream is not None else _null_ctx()):
            ws.zero_()
    _workspaces[key] = (ws, shape)
    return ws


def _fwd_args(q, k, v, idx, softmax_scale, out, lse, stream):
    assert q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    assert v.shape == k.shape and k.shape[:2] == q.shape[:2] and k.shape[3] == q.shape[3]
    assert k.dtype == q.dtype and v.dtype == q.dtype
    B, H, N, d = q.shape
    Nk = k.shape[2]
    assert idx.N == N and (idx.N if idx.Nk is None else idx.Nk) == Nk, "the index was built for a mask of another size"
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    ctx = torch.cuda.stream(stream) if stream is not None else _null_ctx()
    with ctx:                                   # temporaries belong to the stream the kernels run on
        if out is None:
            out = torch.empty_like(q)
        if lse is None:
            lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    return B, H, N, Nk, d, softmax_scale, out, lse


class _null_ctx:
    def __enter__(self):
        return self

    def __exit__(self, *a):
        return False


def bbm_attn_fwd_rect(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx: BlockIndex, mode: int = BBM_MODE_AUTO,
                      softmax_scale: Optional[float] = None, out: Optional[torch.Tensor] = None,
                      lse: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """q: bf16 CUDA tensor [B,H,Nq,d], k, v: [B,H,Nk,d], contiguous.  Returns (O bf16 [B,H,Nq,d], lse fp32 [B,H,Nq]).
    Equal Nq and Nk go through the square entry point of the library."""
    B, H, N, Nk, d, softmax_scale, out, lse = _fwd_args(q, k, v, idx, softmax_scale, out, lse, stream)
    need = bbm_attn_fwd_workspace_bytes(B, H, N, d, idx.Br, idx.Bc, mode)
    if workspace is None and need > 0:
        workspace = _cached_workspace("fwd", need, q.device, stream, (B, H, N, d, idx.Br))
    cs = idx.c_struct()
    ws_bytes = 0 if workspace is None else workspace.numel()
    if Nk == N:
        _check(lib.bbm_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, N, d, softmax_scale, idx.Mb,
                                _ptr(idx.packed_mask), C.byref(cs), mode, _ptr(workspace), ws_bytes, _stream(stream)))
    else:
        _check(lib.bbm_attn_fwd_rect(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, N, Nk, d, softmax_scale, idx.Mb,
                                     _ptr(idx.packed_mask), C.byref(cs), mode, _ptr(workspace), ws_bytes, _stream(stream)))
    return out, lse


def bbm_attn_fwd_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx: BlockIndex, out: torch.Tensor,
                        lse: torch.Tensor, mode: int = BBM_MODE_AUTO, softmax_scale: Optional[float] = None, stream=None):
    """bbm_attn_fwd_rect without a workspace: the library's own static scratch serves LIST mode.  Nothing is allocated
    here either: the caller passes out and lse."""
    B, H, N, Nk, d, softmax_scale, out, lse = _fwd_args(q, k, v, idx, softmax_scale, out, lse, stream)
    cs = idx.c_struct()
    _check(lib.bbm_attn_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, N, Nk, d, softmax_scale, idx.Mb,
                                   _ptr(idx.packed_mask), C.byref(cs), mode, _stream(stream)))
    return out, lse


def bbm_attn_bwd_workspace_bytes(B, H, N, d, Br) -> int:
    return int(lib.bbm_attn_bwd_workspace_bytes(B, H, N, d, Br))


def bbm_attn_bwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, o: torch.Tensor, d_o: torch.Tensor,
                 lse: torch.Tensor, idx: BlockIndex, softmax_scale: Optional[float] = None,
                 dq: Optional[torch.Tensor] = None, dk: Optional[torch.Tensor] = None,
                 dv: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """q, k, v, o, d_o: bf16 CUDA tensors [B,H,N,d], contiguous; lse fp32 [B,H,N] from bbm_attn_fwd; idx built with
    the column list.  Returns (dQ, dK, dV), bf16 [B,H,N,d]."""
    for t in (q, k, v, o, d_o):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape == q.shape
    B, H, N, d = q.shape
    assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.shape == (B, H, N)
    assert idx.N == N and idx.Nk in (None, N), "the index was built for a mask of another size"
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    with (torch.cuda.stream(stream) if stream is not None else _null_ctx()):
        dq = torch.empty_like(q) if dq is None else dq
        dk = torch.empty_like(q) if dk is None else dk
        dv = torch.empty_like(q) if dv is None else dv
    if workspace is None:   # the library wants its counters zero-filled once
        workspace = _cached_workspace("bwd", bbm_attn_bwd_workspace_bytes(B, H, N, d, idx.Br), q.device, stream, (B, H, N, d, idx.Br))
    cs = idx.c_struct()
    _check(lib.bbm_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv),
                            B, H, N, d, softmax_scale, idx.Mb, _ptr(idx.packed_mask), C.byref(cs), _ptr(workspace),
                            workspace.numel(), _stream(stream)))
    return dq, dk, dv


def bbm_rcm_workspace_bytes(N: int) -> int:
    return int(lib.bbm_rcm_workspace_bytes(N))


def bbm_rcm_order(mask2d: torch.Tensor, perm: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                  stream=None) -> torch.Tensor:
    """mask2d: uint8 CUDA tensor [N,N] (row stride may exceed N).  Returns perm int32 [N]: old index of the node at
    each new position (reverse Cuthill-McKee)."""
    assert mask2d.is_cuda and mask2d.dtype == torch.uint8 and mask2d.dim() == 2 and mask2d.stride(1) == 1
    N = mask2d.shape[0]
    assert mask2d.shape[1] == N
    if perm is None:
        perm = torch.empty(N, dtype=torch.int32, device=mask2d.device)
    if workspace is None:
        workspace = torch.empty(max(16, bbm_rcm_workspace_bytes(N)), dtype=torch.uint8, device=mask2d.device)
    _check(lib.bbm_rcm_order(_ptr(mask2d), N, mask2d.stride(0), _ptr(perm), _ptr(workspace), workspace.numel(),
                             _stream(stream)))
    return perm


def bbm_permute_mask(mask: torch.Tensor, perm: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None):
    """mask: uint8 CUDA tensor [Mb,N,N]; returns mask[:, perm][:, :, perm] as a new contiguous tensor."""
    assert mask.is_cuda and mask.dtype == torch.uint8 and mask.dim() == 3 and mask.stride(2) == 1
    Mb, N, _ = mask.shape
    assert mask.shape[2] == N and (Mb == 1 or mask.stride(0) == N * mask.stride(1))
    assert perm.dtype == torch.int32 and perm.is_contiguous() and perm.numel() == N
    if out is None:
        out = torch.empty((Mb, N, N), dtype=torch.uint8, device=mask.device)
    _check(lib.bbm_permute_mask(_ptr(mask), Mb, N, mask.stride(1), _ptr(perm), _ptr(out), _stream(stream)))
    return out


def bbm_gather_rows(x: torch.Tensor, perm: torch.Tensor, inverse: bool = False, out: Optional[torch.Tensor] = None,
                    stream=None) -> torch.Tensor:
    """x: bf16 CUDA tensor [B,H,N,d] contiguous.  inverse=False: out[.., k, :] = x[.., perm[k], :]; True: the scatter."""
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.is_contiguous() and x.dim() == 4
    B, H, N, d = x.shape
    assert perm.dtype == torch.int32 and perm.is_contiguous() and perm.numel() == N
    if out is None:
        out = torch.empty_like(x)
    _check(lib.bbm_gather_rows(_ptr(x), _ptr(perm), _ptr(out), B * H, N, d, 1 if inverse else 0, _stream(stream)))
    return out


def bbm_probe_mfma_bf16(normal_operands: bool, iters: int, sink: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Launches the matrix-instruction-only probe kernel (a measurement aid; the caller times it).  sink: float32 CUDA
    tensor of at least 65536 elements (allocated if None); returned."""
    if sink is None:
        sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.is_contiguous() and sink.numel() >= 65536
    _check(lib.bbm_probe_mfma_bf16(1 if normal_operands else 0, int(iters), _ptr(sink), _stream(stream)))
    return sink


def bbm_probe_mfma_bf16_flop(iters: int) -> float:
    return float(lib.bbm_probe_mfma_bf16_flop(int(iters)))
