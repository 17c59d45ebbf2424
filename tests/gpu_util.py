"""Helpers for the GPU parity tests: move seeded numpy inputs to the device and bring results back."""
import numpy as np
import torch

import oracle


def bf16_tensor(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 CUDA tensor holding the identical bits."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_result_to_f64(t: torch.Tensor) -> np.ndarray:
    bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return oracle.bf16_bits_to_f64(bits)


def index_to_numpy(idx):
    out = {}
    for name in ("blk_class", "bin_blk_mat", "offset", "total_ones", "nz_lo", "nz_hi", "nz_cnt", "row_ptr", "col_ptr"):
        t = getattr(idx, name)
        out[name] = None if t is None else t.cpu().numpy()
    out["col_idx"] = None if idx.col_idx is None else idx.col_idx.cpu().numpy().view(np.uint32)
    out["row_idx"] = None if idx.row_idx is None else idx.row_idx.cpu().numpy().view(np.uint32)
    out["sched"] = None if idx.sched is None else idx.sched.cpu().numpy()
    out["col_sched"] = None if idx.col_sched is None else idx.col_sched.cpu().numpy()
    out["packed_mask"] = None if idx.packed_mask is None else idx.packed_mask.cpu().numpy().view(np.uint64)
    return out


def assert_index_equal(got: dict, mask: np.ndarray, Br: int, Bc: int):
    """Bit-exact comparison of everything the preprocessing stage wrote against the oracle."""
    want = oracle.block_index(mask, Br, Bc)
    assert np.array_equal(got["blk_class"], want["cls"])
    if got["bin_blk_mat"] is not None:
        assert np.array_equal(got["bin_blk_mat"], want["bin_blk_mat"])
    for name in ("offset", "total_ones", "nz_lo", "nz_hi", "nz_cnt"):
        if got[name] is not None:
            assert np.array_equal(got[name], want[name]), name
    if got["row_ptr"] is not None:
        assert np.array_equal(got["row_ptr"], want["row_ptr"])
        Mb, nbr, nbc = want["cls"].shape
        for m in range(Mb):
            n = int(want["row_ptr"][m, -1])
            lo = m * nbr * nbc
            assert np.array_equal(got["col_idx"][lo:lo + n], want["col_idx"][lo:lo + n])
    if got.get("sched") is not None:
        n = oracle.blocks.SCHED_PART_BASE + oracle.blocks.SCHED_PART_INTS * int(want["sched"][0])
        assert np.array_equal(got["sched"][:n], want["sched"][:n])
        Mb, nbr, _ = want["cls"].shape
        assert np.array_equal(got["sched"][-4 * Mb * nbr:], want["sched"][-4 * Mb * nbr:])       # longest-first row records
    if got.get("col_ptr") is not None:
        assert np.array_equal(got["col_ptr"], want["col_ptr"])
        Mb, nbr, nbc = want["cls"].shape
        for m in range(Mb):
            n = int(want["col_ptr"][m, -1])
            lo = m * nbr * nbc
            assert np.array_equal(got["row_idx"][lo:lo + n], want["row_idx"][lo:lo + n])
    if got.get("col_sched") is not None:
        n = oracle.blocks.SCHED_PART_BASE + oracle.blocks.SCHED_PART_INTS * int(want["col_sched"][0])
        assert got["col_sched"].size == want["col_sched"].size and np.array_equal(got["col_sched"][:n], want["col_sched"][:n])
        Mb, _, nbc = want["cls"].shape
        assert np.array_equal(got["col_sched"][-4 * Mb * nbc:], want["col_sched"][-4 * Mb * nbc:])     # launch-order records
    if got["packed_mask"] is not None:
        assert np.array_equal(got["packed_mask"], oracle.packed_bits(mask))


# Tolerances for bf16 inputs/outputs against the fp64 oracle (max-abs, mean-abs on O; max-abs on finite lse).
# lse: the kernel multiplies Q by scale*log2(e) and rounds it to bf16 once per block row (relative error <= 2^-9 per
# element), which moves a score by at most 2^-9 * scale * sum_d |q_d k_d| (about 0.64 * sqrt(d) * 2^-9 = 1.0e-2 / 1.4e-2
# for N(0,1) inputs at d = 64 / 128 if every rounding error had the same sign; a few 1e-3 in practice), and lse moves by
# no more than the largest score error; the row sum adds bf16-rounded probabilities (<= 2^-9 relative, 2e-3).
O_MAX_ABS, O_MEAN_ABS, LSE_MAX_ABS = 2e-2, 2e-3, 1.6e-2


def assert_attention_close(o_gpu: torch.Tensor, lse_gpu: torch.Tensor, O_ref: np.ndarray, lse_ref: np.ndarray):
    o = bf16_result_to_f64(o_gpu)
    l = lse_gpu.cpu().numpy().astype(np.float64)
    assert not np.isnan(o).any() and not np.isnan(l).any()
    err = np.abs(o - O_ref)
    assert err.max() <= O_MAX_ABS, f"max-abs {err.max()}"
    assert err.mean() <= O_MEAN_ABS, f"mean-abs {err.mean()}"
    fin = np.isfinite(lse_ref)
    assert np.array_equal(np.isfinite(l), fin)
    assert np.all(l[~fin] == -np.inf)
    if fin.any():
        assert np.abs(l[fin] - lse_ref[fin]).max() <= LSE_MAX_ABS
    return err.max(), err.mean()


# Gradients (bf16 outputs against the fp64 oracle).  The forward bar (2e-2 max-abs, 2e-3 mean-abs) is stated for O, a
# convex combination of N(0,1) values; dQ, dK, dV are sums over keys resp. queries whose magnitude grows with the
# number of terms, and every error source is relative to the terms (bf16 rounding of P, dS and of the result: 2^-9
# each; the rounding of Q*scale*log2(e) resp. K*scale*log2(e), which moves a probability by up to about 1 %).  So
# the same two bars are applied relative to the size of the tensor: G = max(1, max |reference|).
def assert_grad_close(name: str, got_f64: np.ndarray, ref: np.ndarray):
    assert not np.isnan(got_f64).any(), name
    G = max(1.0, float(np.abs(ref).max()))
    err = np.abs(got_f64 - ref)
    assert err.max() <= O_MAX_ABS * G, f"{name}: max-abs {err.max()} at scale {G}"
    assert err.mean() <= O_MEAN_ABS * G, f"{name}: mean-abs {err.mean()} at scale {G}"
    return err.max(), err.mean()
