#!/usr/bin/env python3
"""Benchmark of the Binary Block Masking forward path on one MI355X.

One "step" is one pass of the whole hot path over one batch: mask -> block classes / BinBlkMat / packed bits
-> run index -> sparse block list -> fused masked attention forward.  Inputs are synthetic, seeded and already
resident in HBM when the timed region starts.

The metric is per mask, so the default run measures every workload of the task (C1..C5), the all-ones and causal
masks at d = 64 and d = 128 (the "dense/causal" case), and reports one row each under `per_mask`.  The headline
(`value`, `config.workload`, `roofline`, `cpu_baseline`) is the largest single-GPU configuration, C5: the reordered
graph mask, B=1 H=8 N=32768 d=64.

Cache regime.  Every timed loop relaunches the same kernel over the same buffers, so whatever fits the chip's
256 MB last-level cache (C1, C2/C0d/C0c: 134 MB of Q/K/V/O; C2's 64 MiB of mask) is served from it after the first
launch: those `*_ms` are warm-cache figures.  Each row therefore also carries `attn_cold_ms` (and
`preprocess_cold_ms`): the same launches rotating over `cold_copies` separate copies of the tensors, sized so that
one round touches more than 768 MB before a buffer is touched again.

Prints ONE JSON line.  `value` = visited-tile TFLOP/s of the whole step (4*Br*Bc*d flops per visited tile per
(batch, head)); `roofline` prices the attention kernel of the headline workload against the roof its algorithmic
intensity puts it under; `cpu_baseline` times the fp64 CPU oracle on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
HBM_PEAK_GBS = 8000.0              # MI355X HBM3E
COLD_BYTES = 768 << 20             # a cold round touches at least this much before a buffer is reused

DEFAULT_MASKS = ["C5", "C1", "C2", "C3", "C4", "C0d", "C0c", "C0d128", "C0c128"]
EXTRA_MASKS = ["C2b", "C4w", "C4d", "C3q", "C3qL", "C5g", "C0d128:256", "C0c128:256"]
DESCRIPTION = {
    "C1": "tiny random-block mask B=1 H=2 N=256 d=64",
    "C2": "packed-sequence mask B=4 H=16 N=4096 d=64 Mb=4",
    "C3": "tree-verification mask B=8 H=32 N=1280 d=128",
    "C4": "long-context sparse pattern B=1 H=16 N=16384 d=64",
    "C5": "reordered graph mask B=1 H=8 N=32768 d=64",
    "C0d": "all-ones mask B=4 H=16 N=4096 d=64", "C0c": "causal mask B=4 H=16 N=4096 d=64",
    "C0d128": "all-ones mask B=2 H=32 N=8192 d=128", "C0c128": "causal mask B=2 H=32 N=8192 d=128",
}


def roofline(kernel: str, algo_flops: float, algo_bytes: float, ms: float, traffic):
    """The roof that bounds a kernel is decided by its algorithmic intensity against the ridge of the two peaks
    (2500 TFLOP/s bf16 MFMA over 8000 GB/s HBM = 312.5 flop/byte); both fractions are reported either way."""
    sec = ms * 1e-3
    tflops, gbs = algo_flops / sec / 1e12, algo_bytes / sec / 1e9
    intensity, ridge = algo_flops / algo_bytes, MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    hbm = intensity < ridge
    return {"bound": "hbm" if hbm else "mfma", "kernel": kernel, "achieved": gbs if hbm else tflops,
            "peak": HBM_PEAK_GBS if hbm else MFMA_BF16_PEAK_TFLOPS, "unit": "GB/s" if hbm else "TFLOP/s",
            "frac": gbs / HBM_PEAK_GBS if hbm else tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
            "algo_bytes": algo_bytes, "algo_flops": algo_flops, "intensity_flop_per_byte": intensity,
            "ridge_flop_per_byte": ridge, "mfma_frac": tflops / MFMA_BF16_PEAK_TFLOPS, "hbm_frac": gbs / HBM_PEAK_GBS,
            "avg_launch_ms": ms}


def profiled_traffic_bytes(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE, each scaled by the
    copy-kernel factor), or None if no summary exists for this kernel and workload."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}.md")
    try:
        for line in open(path):
            if line.startswith("Total traffic per launch:"):
                return float(line.split(":")[1].split("MB")[0]) * 1e6
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C5", help="the headline workload (value, roofline, cpu_baseline)")
    ap.add_argument("--Br", type=int, default=128)
    ap.add_argument("--masks", default="default",
                    help="comma list of workloads reported under per_mask besides the headline: 'default' "
                         f"({','.join(DEFAULT_MASKS)}), 'all' (default plus {','.join(EXTRA_MASKS)}), 'none', or names")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip the backward pass (column list + dQ and dK/dV kernels), which is otherwise timed per mask and "
                         "reported beside the forward figures; the headline value is the forward step either way")
    ap.add_argument("--no-cold", action="store_true", help="skip the rotating-buffer (cold cache) timings")
    ap.add_argument("--only-kernel", default="",
                    help="profile helper: run only 'attn', 'dense' (dense-tile baseline), 'bwd', 'preprocess', 'index' or "
                         "'copy' (256 MiB device copy) launches of --workload")
    ap.add_argument("--scaling", action="store_true",
                    help="instead of the benchmark line: attention time against the number of non-zero blocks, for a window "
                         "mask of fixed width (blocks grow like N) and the causal mask (blocks grow like N^2) at several N")
    ap.add_argument("--operands", action="store_true",
                    help="instead of the benchmark: the matrix-only probe and the dense attention kernel on normal, four-valued and "
                         "constant operands (how much of the gap to the published peak is the chip's clock under load)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured ceilings (matrix-only probe, device copy)")
    ap.add_argument("--B", type=int, default=0, help="with --only-kernel: override the workload's batch size")
    ap.add_argument("--H", type=int, default=0, help="with --only-kernel: override the workload's head count")
    return ap.parse_args()


def time_gpu(fn, warmup, steps):
    """Mean milliseconds per call, HIP events on the current stream (the one the binding launches on) around `steps`
    back-to-back calls."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_gpu_rotating(fns, warmup, steps):
    """As time_gpu, with call n going to fns[n % len(fns)]: closures over separate copies of the buffers."""
    state = {"n": 0}

    def fn():
        fns[state["n"] % len(fns)]()
        state["n"] += 1

    return time_gpu(fn, warmup, max(steps, len(fns)))


def visited_tiles(idx, B, H):
    """Sum over (batch, head, block row) of the number of tiles the schedule visits."""
    per_plane = idx.nz_cnt.sum(dim=1).cpu().numpy().astype(np.int64)     # [Mb]
    per_batch = per_plane if idx.Mb == B else np.repeat(per_plane, B)
    return int(per_batch.sum()) * H


def measure_mask(bbm, name, Br, warmup, steps, torch, backward=False, cold=True):
    from workloads import make_config
    label = name
    if ":" in name:                      # "C0d128:256": this mask at another tile height than --Br
        name, br = name.split(":")
        Br = int(br)
    cfg = make_config(name)
    B, H, N, d, Mb = cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["Mb"]
    Nq = cfg.get("Nq", N)                 # queries per head (N keys): differs only for the decode-time configuration
    backward = backward and Nq == N       # the backward entry point takes one sequence length
    mask = torch.from_numpy(cfg["mask"]).cuda()
    q, k, v = (bbm.bf16_from_bits(cfg[x]) for x in "qkv")
    reorder = None
    if cfg.get("gpu_reorder"):
        # the mask arrives with scrambled node labels (paper Sec. 4, RCM): ordering, permuted mask and gathered Q/K/V
        # are computed on the GPU and timed as a stage of their own; everything below runs on the reordered problem
        blocks_before = int((bbm.bbm_build_block_mask(mask, Br, 64, want_bin=False, want_packed=False).blk_class != 0).sum())
        perm = torch.empty(N, dtype=torch.int32, device="cuda")
        ws_r = torch.empty(bbm.bbm_rcm_workspace_bytes(N), dtype=torch.uint8, device="cuda")
        pm, qg, kg, vg = torch.empty_like(mask), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

        def reorder_stage():
            bbm.bbm_rcm_order(mask[0], perm=perm, workspace=ws_r)
            bbm.bbm_permute_mask(mask, perm, out=pm)
            for src, dst in ((q, qg), (k, kg), (v, vg)):
                bbm.bbm_gather_rows(src, perm, out=dst)

        r_steps = max(2, min(steps, 5))
        reorder = dict(reorder_ms=time_gpu(reorder_stage, 1, r_steps),
                       rcm_order_ms=time_gpu(lambda: bbm.bbm_rcm_order(mask[0], perm=perm, workspace=ws_r), 1, r_steps),
                       blocks_before_reorder=blocks_before)
        mask, q, k, v = pm, qg, kg, vg
        del ws_r
    idx = bbm.build_index(mask, Br, 64)
    out = torch.empty_like(q)
    lse = torch.empty((B, H, Nq), dtype=torch.float32, device="cuda")
    ws = torch.zeros(max(16, bbm.bbm_attn_fwd_workspace_bytes(B, H, Nq, d, Br, 64, bbm.BBM_MODE_LIST)), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    tiles = visited_tiles(idx, B, H)
    cls = idx.blk_class
    census = dict(empty=int((cls == 0).sum()), partial=int((cls == 1).sum()), full=int((cls == 2).sum()))
    flops = 4.0 * Br * 64 * d * tiles
    dense_flops = 4.0 * Nq * N * d * B * H
    useful_flops = 4.0 * float(np.count_nonzero(cfg["mask"])) * (B // Mb) * d * H

    def step():
        bbm.bbm_build_block_mask_rect(mask, Br, 64, idx=idx)
        bbm.bbm_build_index(idx)
        bbm.bbm_attn_fwd_rect(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws)

    res = dict(workload=label, B=B, H=H, N=N, Nq=Nq, d=d, Mb=Mb, Br=Br, Bc=64, visited_tiles=tiles, blocks=census,
               visited_tflop=flops / 1e12, dense_tflop=dense_flops / 1e12, useful_tflop=useful_flops / 1e12)
    if reorder:
        res.update(reorder)
    res["step_ms"] = time_gpu(step, warmup, steps)
    # the same step recorded once into a HIP graph and replayed: what a caller whose mask changes every step (paper
    # Sec. 4: the block matrix of a dynamic mask is rebuilt per step) pays without the three launches' host cost
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    res["graph_step_ms"] = time_gpu(graph.replay, warmup, steps)
    del graph
    for mode_name in ("LIST", "RUNS", "BITMAP"):
        mode = getattr(bbm, "BBM_MODE_" + mode_name)
        ms = time_gpu(lambda: bbm.bbm_attn_fwd_rect(q, k, v, idx, mode=mode, out=out, lse=lse, workspace=ws), warmup, steps)
        res[f"attn_{mode_name.lower()}_ms"] = ms
    res["attn_ms"] = res["attn_list_ms"]
    res["attn_tflops_visited"] = flops / (res["attn_ms"] * 1e-3) / 1e12
    res["attn_mfma_frac"] = res["attn_tflops_visited"] / MFMA_BF16_PEAK_TFLOPS
    dense_steps = max(3, min(steps, int(2000.0 / max(1.0, dense_flops / 1e12 / 0.1))))
    res["dense_tile_ms"] = time_gpu(
        lambda: bbm.bbm_attn_fwd_rect(q, k, v, idx, mode=bbm.BBM_MODE_DENSE_BASELINE, out=out, lse=lse), 2, dense_steps)
    res["dense_tile_tflops"] = dense_flops / (res["dense_tile_ms"] * 1e-3) / 1e12
    res["dense_tile_mfma_frac"] = res["dense_tile_tflops"] / MFMA_BF16_PEAK_TFLOPS
    res["speedup_vs_dense_tile"] = res["dense_tile_ms"] / res["attn_ms"]
    pre_ms = time_gpu(lambda: bbm.bbm_build_block_mask_rect(mask, Br, 64, idx=idx), warmup, steps)
    # algorithmic bytes of the block reduction: every mask byte read once; class and BinBlkMat bytes; the packed words of
    # the non-zero blocks (those of empty blocks are not written)
    nonzero_blocks = int((idx.blk_class != 0).sum())
    pre_bytes = 1.0 * Mb * Nq * N + 2.0 * Mb * idx.nbr * idx.nbc + 8.0 * Br * nonzero_blocks
    res["preprocess_ms"] = pre_ms
    res["preprocess_gbs"] = pre_bytes / (pre_ms * 1e-3) / 1e9
    res["preprocess_hbm_frac"] = res["preprocess_gbs"] / HBM_PEAK_GBS
    res["index_ms"] = time_gpu(lambda: bbm.bbm_build_index(idx), warmup, steps)
    # algorithmic HBM bytes of the attention kernel: Q, K, V read once, O written once, lse, packed words of partial tiles
    res["attn_algo_bytes"] = 2.0 * B * H * (Nq + N) * d * 2 + 4.0 * B * H * Nq + census["partial"] * (B // Mb) * Br * 8.0
    if cold:
        # cold cache: rotate over separate copies of Q/K/V/O/lse (the index and the packed mask are shared by heads,
        # layers and calls, so they stay) resp. of the mask and the preprocessing outputs
        qkvo_bytes = 2.0 * B * H * (Nq + N) * d * 2
        n_att = int(min(8, max(2, math.ceil(COLD_BYTES / qkvo_bytes))))
        sets = [(q, k, v, out, lse)] + [tuple(torch.empty_like(t).copy_(t) for t in (q, k, v, out, lse)) for _ in range(n_att - 1)]
        fns = [(lambda s=s: bbm.bbm_attn_fwd_rect(s[0], s[1], s[2], idx, mode=bbm.BBM_MODE_AUTO, out=s[3], lse=s[4], workspace=ws))
               for s in sets]
        res["attn_cold_ms"] = time_gpu_rotating(fns, n_att, steps)
        res["attn_cold_copies"] = n_att
        res["attn_cold_hbm_frac"] = res["attn_algo_bytes"] / (res["attn_cold_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
        del sets, fns
        mask_bytes = float(Mb) * Nq * N
        if mask_bytes < COLD_BYTES:
            n_pre = int(min(8, max(2, math.ceil(COLD_BYTES / mask_bytes))))
            import copy
            psets = [(mask, idx)]
            for _ in range(n_pre - 1):
                i2 = copy.copy(idx)
                i2.blk_class, i2.bin_blk_mat, i2.packed_mask = (torch.empty_like(t) for t in (idx.blk_class, idx.bin_blk_mat, idx.packed_mask))
                psets.append((mask.clone(), i2))
            pfns = [(lambda s=s: bbm.bbm_build_block_mask_rect(s[0], Br, 64, idx=s[1])) for s in psets]
            res["preprocess_cold_ms"] = time_gpu_rotating(pfns, n_pre, steps)
            res["preprocess_cold_copies"] = n_pre
            res["preprocess_cold_gbs"] = pre_bytes / (res["preprocess_cold_ms"] * 1e-3) / 1e9
            del psets, pfns
        else:
            res["preprocess_cold_ms"], res["preprocess_cold_copies"] = pre_ms, 1     # the mask alone exceeds the cache
            res["preprocess_cold_gbs"] = res["preprocess_gbs"]
    if backward:
        # backward pass: 5 products per visited tile are needed (S, dP, dV, dK, dQ); the two-kernel split executes 7
        # (S and dP are recomputed by both kernels)
        d_o = bbm.bf16_from_bits(cfg["q"][..., ::-1].copy())             # any seeded bf16 tensor of the right shape
        dq, dk, dv = (torch.empty_like(q) for _ in range(3))
        ws_b = torch.zeros(bbm.bbm_attn_bwd_workspace_bytes(B, H, N, d, Br), dtype=torch.uint8, device="cuda")
        bbm.bbm_build_col_index(idx)
        bbm.bbm_attn_fwd(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws)
        res["col_index_ms"] = time_gpu(lambda: bbm.bbm_build_col_index(idx), warmup, steps)
        res["bwd_ms"] = time_gpu(lambda: bbm.bbm_attn_bwd(q, k, v, out, d_o, lse, idx, dq=dq, dk=dk, dv=dv, workspace=ws_b),
                                 warmup, max(3, steps // 2))
        res["bwd_tflops_visited"] = 2.5 * flops / (res["bwd_ms"] * 1e-3) / 1e12
        res["bwd_mfma_frac"] = res["bwd_tflops_visited"] / MFMA_BF16_PEAK_TFLOPS
        res["bwd_executed_tflops"] = 3.5 * flops / (res["bwd_ms"] * 1e-3) / 1e12
        res["fwd_bwd_ms"] = res["attn_ms"] + res["bwd_ms"]
        # algorithmic HBM bytes of the backward pass: Q, K, V, O, dO read once, dQ, dK, dV written once, lse, and the packed
        # words of partial tiles once per kernel
        res["bwd_algo_bytes"] = 8.0 * B * H * N * d * 2 + 4.0 * B * H * N + 2 * census["partial"] * (B // Mb) * Br * 8.0
        res["bwd_hbm_frac"] = res["bwd_algo_bytes"] / (res["bwd_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
        del d_o, dq, dk, dv, ws_b
    # both roofs per workload: the fraction of the HBM peak the algorithmic bytes would need over the kernel's duration,
    # next to the fraction of the MFMA peak; the workload's algorithmic intensity against the ridge names the binding one
    res["attn_hbm_frac"] = res["attn_algo_bytes"] / (res["attn_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    res["attn_intensity_flop_per_byte"] = flops / res["attn_algo_bytes"]
    res["attn_roof"] = "hbm" if res["attn_intensity_flop_per_byte"] < MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS else "mfma"
    res["attn_roof_frac"] = res["attn_hbm_frac"] if res["attn_roof"] == "hbm" else res["attn_mfma_frac"]
    res["attn_traffic_bytes"] = profiled_traffic_bytes("attn_fwd_kernel", name) if Br == 128 else None
    del mask, q, k, v, idx, out, lse, ws
    torch.cuda.empty_cache()
    return res, cfg


def cpu_baseline(cfg, Br, budget_s=20.0, rows_per_chunk=2048):
    """The fp64 oracle, as it stands, on a bounded sample of the headline workload: slabs of `rows_per_chunk` query rows
    (whole block rows) of (batch entry, head) slices, slice by slice, until the time budget is used up.  Each slab
    pays the oracle's block index of its own mask rows and its dense masked attention against all keys."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    N, d, H, B = cfg["N"], cfg["d"], cfg["H"], cfg["B"]
    Nq = cfg.get("Nq", N)
    Mb = cfg["mask"].shape[0]
    rows_per_chunk = max(Br, rows_per_chunk // Br * Br)
    slabs, rows_done, flops, t_idx, t_attn = 0, 0, 0.0, 0.0, 0.0
    done = False
    for b in range(B):
        for h in range(H):
            for r0 in range(0, Nq, rows_per_chunk):
                if t_idx + t_attn >= budget_s:
                    done = True
                    break
                r1 = min(Nq, r0 + rows_per_chunk)
                mask = cfg["mask"][b if Mb == B else 0][None, r0:r1]
                t0 = time.perf_counter()
                idx = oracle.block_index(mask, Br, 64)
                t1 = time.perf_counter()
                oracle.masked_attention(cfg["q"][b:b + 1, h:h + 1, r0:r1], cfg["k"][b:b + 1, h:h + 1], cfg["v"][b:b + 1, h:h + 1], mask)
                t2 = time.perf_counter()
                t_idx += t1 - t0
                t_attn += t2 - t1
                slabs += 1
                rows_done += r1 - r0
                flops += 4.0 * Br * 64 * d * int(idx["nz_cnt"].sum())
            if done:
                break
        if done:
            break
    return dict(value=flops / (t_idx + t_attn) / 1e12 if slabs else 0.0, unit="TFLOP/s (visited tiles)", cores=int(threads), kind="oracle",
                sample=f"{slabs} slabs of up to {rows_per_chunk} query rows = {rows_done} of {B * H * Nq} (batch, head, query) rows of "
                       f"{cfg['name']} (N={N}, d={d}): block index of the slab's mask rows ({t_idx:.2f} s) + dense fp64 masked "
                       f"attention against all {N} keys ({t_attn:.2f} s)",
                seconds=t_idx + t_attn, host_cpus=os.cpu_count())


def only_kernel(a, bbm, torch):
    """Helper for rocprofv3 runs: a plain loop of one kernel on --workload (optionally with fewer heads, so that
    per-dispatch hardware counters of long kernels stay inside their 32-bit range)."""
    from workloads import make_config
    over = {k: v for k, v in (("B", a.B), ("H", a.H)) if v > 0}
    cfg = make_config(a.workload, **over)
    if "B" in over and cfg["Mb"] > 1:
        raise SystemExit("--B cannot be overridden for a workload with one mask per batch entry")
    mask = torch.from_numpy(cfg["mask"]).cuda()
    square = cfg.get("Nq", cfg["N"]) == cfg["N"]
    idx = bbm.build_index(mask, a.Br, 64, columns=square)
    q, k, v = (bbm.bf16_from_bits(cfg[x]) for x in "qkv")
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    ws = torch.zeros(max(16, bbm.bbm_attn_fwd_workspace_bytes(*q.shape, a.Br, 64, bbm.BBM_MODE_LIST)), dtype=torch.uint8, device="cuda")
    if a.only_kernel == "bwd":
        d_o = bbm.bf16_from_bits(cfg["q"][..., ::-1].copy())
        dq, dk, dv = (torch.empty_like(q) for _ in range(3))
        ws_b = torch.zeros(bbm.bbm_attn_bwd_workspace_bytes(*q.shape, a.Br), dtype=torch.uint8, device="cuda")
    if a.only_kernel == "copy":
        src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").fill_(1)     # 256 MiB copy for counter calibration
        dst = torch.empty_like(src)
    bbm.bbm_attn_fwd_rect(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws)
    torch.cuda.synchronize()
    for _ in range(a.warmup + a.steps):
        if a.only_kernel == "bwd":
            bbm.bbm_attn_bwd(q, k, v, out, d_o, lse, idx, dq=dq, dk=dk, dv=dv, workspace=ws_b)
        elif a.only_kernel == "attn":
            bbm.bbm_attn_fwd_rect(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws)
        elif a.only_kernel == "dense":
            bbm.bbm_attn_fwd_rect(q, k, v, idx, mode=bbm.BBM_MODE_DENSE_BASELINE, out=out, lse=lse)
        elif a.only_kernel == "preprocess":
            bbm.bbm_build_block_mask_rect(mask, a.Br, 64, idx=idx)
        elif a.only_kernel == "index":
            bbm.bbm_build_index(idx)
        elif a.only_kernel == "copy":
            dst.copy_(src)
        else:
            raise SystemExit(f"unknown --only-kernel {a.only_kernel}")
    torch.cuda.synchronize()
    return 0


def scaling_study(a, bbm, torch):
    """Does the run time follow the number of non-zero blocks rather than N^2 (the method's claim, paper Sec. 4)?  One head
    count and head dimension throughout (B=1, H=16, d=64); masks built on the device; Q, K, V seeded normal bf16."""
    B, H, d, Br = 1, 16, 64, a.Br
    rows = []
    for family, sizes in (("window +-256", (2048, 4096, 8192, 16384, 32768)), ("causal", (2048, 4096, 8192, 16384))):
        for N in sizes:
            i = torch.arange(N, device="cuda", dtype=torch.int32)
            mask = torch.empty((1, N, N), dtype=torch.uint8, device="cuda")
            for r0 in range(0, N, 4096):                      # row slabs: the index difference matrix is never whole
                diff = i[r0:r0 + 4096, None] - i[None, :]
                mask[0, r0:r0 + 4096] = ((diff.abs() <= 256) if family.startswith("window") else (diff >= 0)).to(torch.uint8)
            del diff
            gen = torch.Generator(device="cuda").manual_seed(1234 + N)
            q, k, v = (torch.randn((B, H, N, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
            idx = bbm.build_index(mask, Br, 64)
            out = torch.empty_like(q)
            lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
            ws = torch.zeros(max(16, bbm.bbm_attn_fwd_workspace_bytes(B, H, N, d, Br, 64, bbm.BBM_MODE_LIST)), dtype=torch.uint8, device="cuda")
            tiles = visited_tiles(idx, B, H)
            ms = time_gpu(lambda: bbm.bbm_attn_fwd(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws), a.warmup, a.steps)
            dense_ms = time_gpu(lambda: bbm.bbm_attn_fwd(q, k, v, idx, mode=bbm.BBM_MODE_DENSE_BASELINE, out=out, lse=lse), 1, max(2, min(a.steps, 10)))
            pre_ms = time_gpu(lambda: bbm.bbm_build_block_mask(mask, Br, 64, idx=idx), a.warmup, a.steps)
            rows.append(dict(mask=family, N=N, nonzero_blocks=tiles // H, all_blocks=idx.nbr * idx.nbc, attn_ms=ms,
                             us_per_1000_blocks_per_head=ms * 1e3 / (tiles / 1000.0) * H, dense_tile_ms=dense_ms,
                             tflops_visited=4.0 * Br * 64 * d * tiles / (ms * 1e-3) / 1e12, preprocess_ms=pre_ms))
            del mask, q, k, v, idx, out, lse, ws
            torch.cuda.empty_cache()
    print(json.dumps({"study": "attention time against non-zero blocks", "B": B, "H": H, "d": d, "Br": Br, "Bc": 64, "rows": rows}))
    return 0


def measure_ceilings(bbm, torch):
    """What this chip sustains, next to the published figures the roofline is quoted against: matrix instructions
    alone (bbm_probe_mfma_bf16: one wave per SIMD, operands in registers) on constant and on normal operands, and a
    256 MiB device-to-device copy.  Each probe launch is preceded by a shorter one, so the clock has settled."""
    sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    res = {}
    for key, normal in (("mfma_bf16_constant_operands_tflops", False), ("mfma_bf16_normal_operands_tflops", True)):
        bbm.bbm_probe_mfma_bf16(normal, 20000, sink)
        ms = time_gpu(lambda: bbm.bbm_probe_mfma_bf16(normal, 100000, sink), 0, 1)
        res[key] = bbm.bbm_probe_mfma_bf16_flop(100000) / (ms * 1e-3) / 1e12
    src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    ms = time_gpu(lambda: dst.copy_(src), 3, 10)
    res["device_copy_gbs"] = 2.0 * src.numel() / (ms * 1e-3) / 1e9
    return res


def operand_study(a, bbm, torch):
    """The same dense attention launch on three kinds of operands.  The instruction stream is identical; what changes
    is the power the arithmetic units draw, and with it the clock the chip holds."""
    rows = []
    gen = torch.Generator(device="cuda").manual_seed(99)
    kinds = {
        "normal(0,1)": lambda shape: tuple(torch.randn(shape, generator=gen, device="cuda").to(torch.bfloat16) for _ in range(3)),
        "four values (+-0.5, +-1.5)": lambda shape: tuple((torch.randint(0, 4, shape, generator=gen, device="cuda").float() - 1.5).to(torch.bfloat16) for _ in range(3)),
        "constant (0.5, 0.25, 1.0)": lambda shape: tuple(torch.full(shape, c, device="cuda", dtype=torch.bfloat16) for c in (0.5, 0.25, 1.0)),
    }
    for (B, H, N, d) in ((2, 32, 8192, 128), (4, 16, 4096, 64)):
        mask = torch.ones((1, N, N), dtype=torch.uint8, device="cuda")
        idx = bbm.build_index(mask, a.Br, 64)
        out = torch.empty((B, H, N, d), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        ws = torch.zeros(max(16, bbm.bbm_attn_fwd_workspace_bytes(B, H, N, d, a.Br, 64, bbm.BBM_MODE_LIST)), dtype=torch.uint8, device="cuda")
        for kind, make in kinds.items():
            q, k, v = make((B, H, N, d))
            ms = time_gpu(lambda: bbm.bbm_attn_fwd(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws), a.warmup, a.steps)
            rows.append(dict(B=B, H=H, N=N, d=d, operands=kind, attn_ms=ms, tflops=4.0 * B * H * N * N * d / (ms * 1e-3) / 1e12))
        del mask, idx, out, lse, ws, q, k, v
    print(json.dumps({"study": "dense attention forward against the kind of operands", "Br": a.Br, "Bc": 64,
                      "ceilings": measure_ceilings(bbm, torch), "rows": rows}))
    return 0


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (no sharding, no collectives); got --gpus {a.gpus}",
              file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    import paper_2409_15097_amd as bbm

    if a.only_kernel:
        return only_kernel(a, bbm, torch)
    if a.scaling:
        return scaling_study(a, bbm, torch)
    if a.operands:
        return operand_study(a, bbm, torch)

    main_res, main_cfg = measure_mask(bbm, a.workload, a.Br, a.warmup, a.steps, torch, not a.no_backward, not a.no_cold)
    rows = [main_res]
    extra = {"default": DEFAULT_MASKS, "all": DEFAULT_MASKS + EXTRA_MASKS, "none": []}.get(a.masks, a.masks.split(","))
    for name in [m for m in extra if m and m != a.workload]:
        r, _ = measure_mask(bbm, name, a.Br, a.warmup, a.steps, torch, not a.no_backward, not a.no_cold)
        rows.append(r)

    flops = main_res["visited_tflop"] * 1e12
    step_ms = main_res["step_ms"]
    out = {
        "metric": "masked attn fwd ms + TFLOP/s on visited tiles vs dense-tile kernel, per mask",
        "value": flops / (step_ms * 1e-3) / 1e12,
        "unit": "TFLOP/s (visited tiles, whole step: preprocess + index + attention)",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {DESCRIPTION[a.workload]}" if a.workload in DESCRIPTION else a.workload,
                   "Br": a.Br, "Bc": 64, "mode": "AUTO(LIST)",
                   "cache": "warm (same buffers relaunched; working sets under 256 MB stay in the last-level cache); "
                            "*_cold_ms rotate copies beyond 768 MB"},
        "attn_ms": main_res["attn_ms"], "attn_tflops_visited": main_res["attn_tflops_visited"],
        "dense_tile_ms": main_res["dense_tile_ms"], "dense_tile_tflops": main_res["dense_tile_tflops"],
        "preprocess_ms": main_res["preprocess_ms"], "preprocess_gbs": main_res["preprocess_gbs"],
        "graph_step_ms": main_res["graph_step_ms"],
        "roofline": roofline("attn_fwd_kernel", flops, main_res["attn_algo_bytes"], main_res["attn_ms"],
                             profiled_traffic_bytes("attn_fwd_kernel", a.workload)),
        "per_mask": rows,
    }
    if not a.no_backward and "bwd_ms" in main_res:
        # the next step of the path: backward pass over the same block index.  Algorithmic work: 5 products per visited
        # tile (S, dP, dV, dK, dQ) = 2.5 x the forward; the two-kernel split executes 7 (S and dP twice).
        out["backward"] = {
            "bwd_ms": main_res["bwd_ms"], "col_index_ms": main_res["col_index_ms"], "fwd_bwd_ms": main_res["fwd_bwd_ms"],
            "roofline": dict(roofline("attn_bwd_dq_kernel + attn_bwd_dkv_kernel", 2.5 * flops, main_res["bwd_algo_bytes"],
                                      main_res["bwd_ms"], profiled_traffic_bytes("attn_bwd_kernels", a.workload)),
                             executed_tflops=main_res["bwd_executed_tflops"])}
    if not a.no_ceilings:
        # measured on this chip in this run; the roofline above stays priced against the published peaks
        out["ceilings"] = measure_ceilings(bbm, torch)
        if out["roofline"]["bound"] == "mfma":
            out["roofline"]["frac_of_measured_matrix_rate_normal_operands"] = (
                out["roofline"]["achieved"] / out["ceilings"]["mfma_bf16_normal_operands_tflops"])
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(main_cfg, a.Br)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
