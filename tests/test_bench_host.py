"""Host-side logic of bench.py (CPU only): which roof a workload is priced against, the default set of workloads, the
refusal of more than one GPU, and the bounded CPU baseline."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_roof_follows_the_algorithmic_intensity():
    ridge = 2500e12 / 8000e9
    below = bench.roofline("k", algo_flops=100.0 * 1e6, algo_bytes=1e6, ms=1.0, traffic=None)       # 100 flop/byte
    above = bench.roofline("k", algo_flops=1000.0 * 1e6, algo_bytes=1e6, ms=1.0, traffic=2e6)      # 1000 flop/byte
    assert below["bound"] == "hbm" and below["unit"] == "GB/s" and below["peak"] == 8000.0
    assert above["bound"] == "mfma" and above["unit"] == "TFLOP/s" and above["peak"] == 2500.0
    assert abs(below["ridge_flop_per_byte"] - ridge) < 1e-9
    # 1e6 bytes in 1 ms = 1 GB/s; 1e9 flop in 1 ms = 1 TFLOP/s; fractions are achieved / peak of the chosen roof
    assert abs(below["achieved"] - 1.0) < 1e-12 and abs(below["frac"] - 1.0 / 8000.0) < 1e-15
    assert abs(above["achieved"] - 1.0) < 1e-12 and abs(above["frac"] - 1.0 / 2500.0) < 1e-15
    assert above["traffic"] == 2e6 and below["traffic"] is None
    for r in (below, above):
        assert abs(r["mfma_frac"] - r["algo_flops"] / 1e-3 / 1e12 / 2500.0) < 1e-15
        assert abs(r["hbm_frac"] - r["algo_bytes"] / 1e-3 / 1e9 / 8000.0) < 1e-15


def test_default_run_covers_every_workload_of_the_task_and_the_dense_causal_case():
    assert bench.DEFAULT_MASKS[0] == "C5"                      # the headline: the largest single-GPU configuration
    assert set(bench.DEFAULT_MASKS) >= {"C1", "C2", "C3", "C4", "C5", "C0d", "C0c", "C0d128", "C0c128"}
    assert all(m in bench.DESCRIPTION for m in bench.DEFAULT_MASKS)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_cpu_baseline_is_bounded_and_counts_visited_tiles():
    from workloads import make_config
    import oracle
    cfg = make_config("C1")
    res = bench.cpu_baseline(cfg, 128, budget_s=30.0, rows_per_chunk=128)
    assert res["kind"] == "oracle" and res["cores"] >= 1 and res["value"] > 0
    # the whole tiny workload fits the budget: 2 heads x 2 slabs, and the flop count is that of the oracle's own block index
    tiles = int(oracle.block_index(cfg["mask"], 128, 64)["nz_cnt"].sum()) * cfg["H"]
    assert abs(res["value"] * res["seconds"] * 1e12 - 4.0 * 128 * 64 * 64 * tiles) < 1.0
    assert "4 slabs" in res["sample"]
    none = bench.cpu_baseline(cfg, 128, budget_s=0.0)        # no budget: nothing is run, nothing is divided by zero
    assert none["seconds"] == 0.0 and none["value"] == 0.0 and "0 slabs" in none["sample"]
