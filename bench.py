#!/usr/bin/env python3
"""Benchmark of the Binary Block Masking forward path on one MI355X.

One "step" is one pass of the whole hot path over one batch: mask -> block classes / BinBlkMat / packed bits
-> run index -> sparse block list -> fused masked attention forward.  Inputs are synthetic, seeded and already
resident in HBM when the timed region starts.  The headline workload is the packed-sequence mask
(B=4, H=16, N=4096, d=64, one mask per batch entry); the other mask families are timed as extra rows.

Prints ONE JSON line.  `value` = visited-tile TFLOP/s of the whole step (4*Br*Bc*d flops per visited tile per
(batch, head)); `roofline` prices the attention kernel against the bf16 MFMA peak; `cpu_baseline` times the
fp64 CPU oracle on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
HBM_PEAK_GBS = 8000.0              # MI355X HBM3E


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
            "ridge_flop_per_byte": ridge, "mfma_frac": tflops / MFMA_BF16_PEAK_TFLOPS, "hbm_frac": gbs / HBM_PEAK_GBS}


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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--Br", type=int, default=128)
    ap.add_argument("--masks", default="",
                    help="comma list of extra workloads measured the same way and reported under per_mask, or 'all' "
                         "(C3,C4,C5,C0d,C0c,C0d128,C0c128); default: the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip the backward pass (column list + dQ and dK/dV kernels), which is otherwise timed per mask and "
                         "reported beside the forward figures; the headline value is the forward step either way")
    ap.add_argument("--only-kernel", default="", help="profile helper: run only 'attn', 'bwd', 'preprocess' or 'copy' (256 MiB device copy) launches")
    return ap.parse_args()


def time_gpu(fn, warmup, steps):
    """Mean milliseconds per call, HIP events on the current stream around `steps` back-to-back calls."""
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


def visited_tiles(idx, B, H):
    """Sum over (batch, head, block row) of the number of tiles the schedule visits."""
    per_plane = idx.nz_cnt.sum(dim=1).cpu().numpy().astype(np.int64)     # [Mb]
    per_batch = per_plane if idx.Mb == B else np.repeat(per_plane, B)
    return int(per_batch.sum()) * H


def measure_mask(bbm, name, Br, warmup, steps, torch, backward=False):
    from workloads import make_config
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

    res = dict(workload=name, B=B, H=H, N=N, Nq=Nq, d=d, Mb=Mb, Br=Br, Bc=64, visited_tiles=tiles, blocks=census,
               visited_tflop=flops / 1e12, dense_tflop=dense_flops / 1e12, useful_tflop=useful_flops / 1e12)
    if reorder:
        res.update(reorder)
    res["step_ms"] = time_gpu(step, warmup, steps)
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
    res["speedup_vs_dense_tile"] = res["dense_tile_ms"] / res["attn_ms"]
    pre_ms = time_gpu(lambda: bbm.bbm_build_block_mask_rect(mask, Br, 64, idx=idx), warmup, steps)
    pre_bytes = Mb * Nq * N * (1.0 + 1.0 / 8.0) + 2.0 * Mb * idx.nbr * idx.nbc
    res["preprocess_ms"] = pre_ms
    res["preprocess_gbs"] = pre_bytes / (pre_ms * 1e-3) / 1e9
    res["preprocess_hbm_frac"] = res["preprocess_gbs"] / HBM_PEAK_GBS
    res["index_ms"] = time_gpu(lambda: bbm.bbm_build_index(idx), warmup, steps)
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
                                 warmup, steps)
        res["bwd_tflops_visited"] = 2.5 * flops / (res["bwd_ms"] * 1e-3) / 1e12
        res["bwd_mfma_frac"] = res["bwd_tflops_visited"] / MFMA_BF16_PEAK_TFLOPS
        res["bwd_executed_tflops"] = 3.5 * flops / (res["bwd_ms"] * 1e-3) / 1e12
        res["fwd_bwd_ms"] = res["attn_ms"] + res["bwd_ms"]
        # algorithmic HBM bytes of the backward pass: Q, K, V, O, dO read once, dQ, dK, dV written once, lse, and the packed
        # words of partial tiles once per kernel
        res["bwd_algo_bytes"] = 8.0 * B * H * N * d * 2 + 4.0 * B * H * N + 2 * census["partial"] * (B // Mb) * Br * 8.0
        del d_o, dq, dk, dv, ws_b
    # algorithmic HBM bytes of the attention kernel: Q, K, V read once, O written once, lse, packed words of partial tiles
    res["attn_algo_bytes"] = 2.0 * B * H * (Nq + N) * d * 2 + 4.0 * B * H * Nq + census["partial"] * (B // Mb) * Br * 8.0
    # both roofs per workload: the fraction of the HBM peak the algorithmic bytes would need over the kernel's duration,
    # next to the fraction of the MFMA peak; the larger one names the roof the kernel is closer to
    res["attn_hbm_frac"] = res["attn_algo_bytes"] / (res["attn_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    res["attn_nearer_roof"] = "hbm" if res["attn_hbm_frac"] > res["attn_mfma_frac"] else "mfma"
    del mask, q, k, v, idx, out, lse, ws
    torch.cuda.empty_cache()
    return res, cfg


def cpu_baseline(cfg, Br, budget_s=20.0):
    """The fp64 oracle, as it stands, on a bounded sample of the headline workload: whole (batch entry, head) slices,
    batch entry by batch entry, until the time budget is used up (the whole workload if it fits)."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    N, d, H, B = cfg["N"], cfg["d"], cfg["H"], cfg["B"]
    Mb = cfg["mask"].shape[0]
    slices, flops, t_idx, t_attn = 0, 0.0, 0.0, 0.0
    for b in range(B):
        mask = cfg["mask"][b:b + 1] if Mb == B else cfg["mask"][:1]
        t0 = time.perf_counter()
        idx = oracle.block_index(mask, Br, 64)
        t_idx += time.perf_counter() - t0
        tiles_per_head = int(idx["nz_cnt"].sum())
        for h in range(H):
            if t_idx + t_attn >= budget_s:
                break
            t0 = time.perf_counter()
            oracle.masked_attention(cfg["q"][b:b + 1, h:h + 1], cfg["k"][b:b + 1, h:h + 1], cfg["v"][b:b + 1, h:h + 1], mask)
            t_attn += time.perf_counter() - t0
            slices += 1
            flops += 4.0 * Br * 64 * d * tiles_per_head
        if t_idx + t_attn >= budget_s:
            break
    return dict(value=flops / (t_idx + t_attn) / 1e12, unit="TFLOP/s (visited tiles)", cores=int(threads), kind="oracle",
                sample=f"{slices} of {B * H} (batch entry, head) slices of {cfg['name']} (N={N}, d={d}): block index per batch "
                       f"entry ({t_idx:.2f} s) + dense fp64 masked attention ({t_attn:.2f} s)",
                seconds=t_idx + t_attn, host_cpus=os.cpu_count())


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

    if a.only_kernel:                      # helper for rocprofv3 runs: a plain loop of one kernel
        from workloads import make_config
        cfg = make_config(a.workload)
        mask = torch.from_numpy(cfg["mask"]).cuda()
        idx = bbm.build_index(mask, a.Br, 64, columns=True)
        q, k, v = (bbm.bf16_from_bits(cfg[x]) for x in "qkv")
        out = torch.empty_like(q)
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
        d_o = bbm.bf16_from_bits(cfg["q"][..., ::-1].copy())
        dq, dk, dv = (torch.empty_like(q) for _ in range(3))
        ws_b = torch.zeros(bbm.bbm_attn_bwd_workspace_bytes(*q.shape, a.Br), dtype=torch.uint8, device="cuda")
        ws = torch.zeros(max(16, bbm.bbm_attn_fwd_workspace_bytes(*q.shape, a.Br, 64, bbm.BBM_MODE_LIST)), dtype=torch.uint8, device="cuda")
        src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").fill_(1)     # 256 MiB copy for counter calibration
        dst = torch.empty_like(src)
        bbm.bbm_attn_fwd(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws)
        torch.cuda.synchronize()
        for _ in range(a.warmup + a.steps):
            if a.only_kernel == "bwd":
                bbm.bbm_attn_bwd(q, k, v, out, d_o, lse, idx, dq=dq, dk=dk, dv=dv, workspace=ws_b)
            elif a.only_kernel == "attn":
                bbm.bbm_attn_fwd(q, k, v, idx, mode=bbm.BBM_MODE_AUTO, out=out, lse=lse, workspace=ws)
            elif a.only_kernel == "preprocess":
                bbm.bbm_build_block_mask(mask, a.Br, 64, idx=idx)
            elif a.only_kernel == "copy":
                dst.copy_(src)
            else:
                raise SystemExit(f"unknown --only-kernel {a.only_kernel}")
        torch.cuda.synchronize()
        return 0

    main_res, main_cfg = measure_mask(bbm, a.workload, a.Br, a.warmup, a.steps, torch, not a.no_backward)
    rows = [main_res]
    extra = "C3,C4,C5,C0d,C0c,C0d128,C0c128,C2b,C4w,C4d,C3q,C3qL,C5g,C0d128:256,C0c128:256" if a.masks == "all" else a.masks
    for name in [m for m in extra.split(",") if m and m != a.workload]:
        r, _ = measure_mask(bbm, name, a.Br, a.warmup, a.steps, torch, not a.no_backward)
        rows.append(r)

    flops = main_res["visited_tflop"] * 1e12
    step_ms = main_res["step_ms"]
    out = {
        "metric": "masked attn fwd ms + TFLOP/s on visited tiles vs dense-tile kernel, per mask",
        "value": flops / (step_ms * 1e-3) / 1e12,
        "unit": "TFLOP/s (visited tiles, whole step: preprocess + index + attention)",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: packed-sequence mask B=4 H=16 N=4096 d=64 Mb=4" if a.workload == "C2" else a.workload,
                   "Br": a.Br, "Bc": 64, "mode": "AUTO(LIST)"},
        "attn_ms": main_res["attn_ms"], "attn_tflops_visited": main_res["attn_tflops_visited"],
        "dense_tile_ms": main_res["dense_tile_ms"], "dense_tile_tflops": main_res["dense_tile_tflops"],
        "preprocess_ms": main_res["preprocess_ms"], "preprocess_gbs": main_res["preprocess_gbs"],
        "roofline": roofline("attn_fwd_kernel", flops, main_res["attn_algo_bytes"], main_res["attn_ms"],
                             profiled_traffic_bytes("attn_fwd_kernel", a.workload)),
        "per_mask": rows,
    }
    if not a.no_backward:
        # the next step of the path: backward pass over the same block index.  Algorithmic work: 5 products per visited
        # tile (S, dP, dV, dK, dQ) = 2.5 x the forward; the two-kernel split executes 7 (S and dP twice).
        out["backward"] = {
            "bwd_ms": main_res["bwd_ms"], "col_index_ms": main_res["col_index_ms"], "fwd_bwd_ms": main_res["fwd_bwd_ms"],
            "roofline": dict(roofline("attn_bwd_dq_kernel + attn_bwd_dkv_kernel", 2.5 * flops, main_res["bwd_algo_bytes"],
                                      main_res["bwd_ms"], profiled_traffic_bytes("attn_bwd_kernels", a.workload)),
                             executed_tflops=main_res["bwd_executed_tflops"])}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(main_cfg, a.Br)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
