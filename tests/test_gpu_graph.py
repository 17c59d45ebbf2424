"""GPU: the whole step (block reduction, index, attention forward, column list, backward) recorded into a HIP graph and
replayed.  The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
caller may capture it; every replay must reproduce the eager results bit for bit, also with other work in between."""
import numpy as np
import pytest
import torch

from workloads import make_qkv
from gpu_util import bf16_tensor

pytestmark = pytest.mark.gpu


def test_step_replays_from_a_graph_with_eager_work_in_between():
    import paper_2409_15097_amd as bbm
    B, H, N, d, Br = 1, 2, 4096, 64, 128
    i = np.arange(N)
    m = (np.abs(i[:, None] - i[None, :]) <= 70).astype(np.uint8)
    m[300:340] = 1                                         # global query rows and global keys: the schedules cut their
    m[:, 1000:1030] = 1                                    # block row and block column, so the queue counters are exercised
    mask = torch.from_numpy(m[None]).cuda()
    q, k, v = (bf16_tensor(x) for x in make_qkv(B, H, N, d, seed=7))
    d_o = bf16_tensor(make_qkv(B, H, N, d, seed=991)[0])

    def buffers():
        idx = bbm.build_index(mask, Br, 64, columns=True)                      # allocates every index tensor once
        o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
        lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        ws_f = torch.zeros(max(16, bbm.bbm_attn_fwd_workspace_bytes(B, H, N, d, Br, 64, bbm.BBM_MODE_LIST)), dtype=torch.uint8, device="cuda")
        ws_b = torch.zeros(bbm.bbm_attn_bwd_workspace_bytes(B, H, N, d, Br), dtype=torch.uint8, device="cuda")
        return idx, o, lse, dq, dk, dv, ws_f, ws_b

    def step(idx, o, lse, dq, dk, dv, ws_f, ws_b):
        bbm.bbm_build_block_mask(mask, Br, 64, idx=idx)
        bbm.bbm_build_index(idx)
        bbm.bbm_build_col_index(idx)
        bbm.bbm_attn_fwd(q, k, v, idx, out=o, lse=lse, workspace=ws_f)
        bbm.bbm_attn_bwd(q, k, v, o, d_o, lse, idx, dq=dq, dk=dk, dv=dv, workspace=ws_b)

    eager = buffers()
    step(*eager)
    torch.cuda.synchronize()
    assert int(eager[0].sched[0]) > 0 and int(eager[0].col_sched[0]) > 0
    want = [t.clone() for t in (eager[1], eager[2], eager[3], eager[4], eager[5])]

    rec = buffers()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(*rec)                                                               # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(*rec)
    for replay in range(3):
        for t in rec[1:6]:
            t.fill_(float("nan")) if t.is_floating_point() else t.zero_()       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (rec[1], rec[2], rec[3], rec[4], rec[5])
        for name, a, b in zip(("o", "lse", "dq", "dk", "dv"), got, want):
            same = torch.equal(a.view(torch.int16), b.view(torch.int16)) if a.dtype == torch.bfloat16 else torch.equal(a, b)
            assert same, f"replay {replay}: {name} differs from the eager result"
