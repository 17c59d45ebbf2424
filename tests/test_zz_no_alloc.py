"""GPU test of bbm_attn_fwd_static, the forward entry point that allocates nothing: its counters and partial results
live in a static device array of the library instead of a caller's workspace.  Its output is compared with that of
bbm_attn_fwd_rect (caller's workspace) on the same inputs, bit for bit: both run the same kernels with the same
work split whenever the partial results fit the static array, which they do here.  Two calls in a row share the
array, the second with a smaller input; then a small launch whose block rows are computed in parts."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from workloads import make_qkv, small_variant
from gpu_util import bf16_tensor, assert_attention_close

pytestmark = pytest.mark.gpu


def _both(bbm, q, k, v, mask, Br, mode):
    """(O, lse) from the workspace entry point and from the static one, the latter called through ctypes directly."""
    idx = bbm.build_index(torch.from_numpy(np.ascontiguousarray(mask)).cuda(), Br, 64)
    qt, kt, vt = (bf16_tensor(x) for x in (q, k, v))
    B, H, Nq, d = qt.shape
    Nk = kt.shape[2]
    o_ws, lse_ws = bbm.bbm_attn_fwd_rect(qt, kt, vt, idx, mode=mode)
    o_st = torch.full_like(o_ws, float("nan"))
    lse_st = torch.full_like(lse_ws, float("nan"))
    torch.cuda.synchronize()
    cs = idx.c_struct()
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = bbm.lib.bbm_attn_fwd_static(p(qt), p(kt), p(vt), p(o_st), p(lse_st), B, H, Nq, Nk, d, C.c_float(d ** -0.5), idx.Mb,
                                     p(idx.packed_mask), C.byref(cs), mode, C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == bbm.BBM_OK, bbm.bbm_last_error()
    torch.cuda.synchronize()
    return idx, (o_ws, lse_ws), (o_st, lse_st)


def _same_bits(a, b):
    return torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


def test_static_scratch_forward_matches_the_workspace_forward_on_two_calls_in_a_row():
    import paper_2409_15097_amd as bbm
    # call 1: long-context sparse pattern, whose global-token block rows the schedule cuts into parts (the parts'
    # partial results and the queue counters go through the scratch); call 2: the same family, shorter and with fewer heads
    for n_call, (N, H) in enumerate(((4096, 4), (2560, 2))):
        cfg = small_variant("C4", N=N, B=1, H=H)
        print(f"static scratch call {n_call + 1}: C4 family N={N} H={H}", flush=True)
        idx, ws_out, st_out = _both(bbm, cfg["q"], cfg["k"], cfg["v"], cfg["mask"], 128, bbm.BBM_MODE_LIST)
        assert int(idx.sched[0]) >= 2, "the case is meant to have cut rows"
        assert _same_bits(ws_out, st_out)
        O_ref, lse_ref = oracle.masked_attention(cfg["q"], cfg["k"], cfg["v"], cfg["mask"])
        assert_attention_close(st_out[0], st_out[1], O_ref, lse_ref)
    # call 3, smaller again in work-groups: 3 heads x 3 block rows against 16400 keys, every block row in 8 parts
    B, H, d, Nq, Nk = 1, 3, 64, 300, 16400
    q = make_qkv(B, H, Nq, d, seed=41)[0]
    _, k, v = make_qkv(B, H, Nk, d, seed=42)
    mask = (np.random.default_rng(43).random((1, Nq, Nk)) < 0.3).astype(np.uint8)
    mask[0, :, 3000:9000] = 1
    mask[0, 128:192] = 0
    print("static scratch call 3: small launch computed in parts", flush=True)
    _, ws_out, st_out = _both(bbm, q, k, v, mask, 128, bbm.BBM_MODE_AUTO)
    assert _same_bits(ws_out, st_out)
    O_ref, lse_ref = oracle.masked_attention(q, k, v, mask)
    assert_attention_close(st_out[0], st_out[1], O_ref, lse_ref)
    # schedules that use no scratch pass through unchanged
    _, ws_out, st_out = _both(bbm, q, k, v, mask, 128, bbm.BBM_MODE_BITMAP)
    assert _same_bits(ws_out, st_out)
