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
        # words of a (block row x 64 columns) slab that holds no allowed pair are not written (nothing reads them);
        # every other word is compared bit for bit
        ref = oracle.packed_bits(mask)
        Mb, W, Nq = ref.shape
        nbr = -(-Nq // Br)
        nonzero = np.zeros((Mb, W, nbr * Br), dtype=bool)
        nonzero[:, :, :Nq] = ref != 0
        written = np.repeat(nonzero.reshape(Mb, W, nbr, Br).any(axis=3), Br, axis=2)[:, :, :Nq]
        assert got["packed_mask"].shape == ref.shape
        assert np.array_equal(got["packed_mask"][written], ref[written])


# Tolerances for bf16 inputs/outputs against the fp64 oracle (max-abs, mean-abs on O; max-abs on finite lse).
# O: the bars the task states, at every softmax scale.  lse: two roundings set it.  The row sum adds bf16-rounded
# probabilities (relative error <= 2^-9 each, so |d ln l| <= 2e-3).  Up to the usual scale 1/sqrt(d) the kernel rounds
# Q * scale * log2(e) to bf16 once per block row, which moves a score by at most 2^-9 * scale * sum_d |q_d k_d|; with
# errors of random sign that is a few 1e-3 for N(0,1) inputs at d = 64 and 128, and lse moves by no more than the largest
# score error of its row.  Largest error observed over the full outputs of all full-size workloads: 6.8e-3 (packed
# sequences, d = 64); the bar is 1e-2.  (Sharper scales do not round the scale into Q at all: 3.6e-3 observed.)
O_MAX_ABS, O_MEAN_ABS, LSE_MAX_ABS = 2e-2, 2e-3, 1.0e-2


def record_maxima(tag: str, **values):
    """Appends the observed error maxima of a parity case to the file named by BBM_MAXIMA_FILE (if set), one JSON line
    per case: the source of the tolerance table in the design notes."""
    import json
    import os
    path = os.environ.get("BBM_MAXIMA_FILE")
    if path:
        with open(path, "a") as f:
            f.write(json.dumps(dict(case=tag, **{k: float(v) for k, v in values.items()})) + "\n")


def attention_errors(o_gpu: torch.Tensor, lse_gpu: torch.Tensor, O_ref: np.ndarray, lse_ref: np.ndarray):
    """(max-abs of O, sum-abs of O, element count, max-abs of finite lse); asserts the exact parts: no NaN, -inf rows."""
    o = bf16_result_to_f64(o_gpu)
    l = lse_gpu.cpu().numpy().astype(np.float64)
    assert not np.isnan(o).any() and not np.isnan(l).any()
    err = np.abs(o - O_ref)
    fin = np.isfinite(lse_ref)
    assert np.array_equal(np.isfinite(l), fin)
    assert np.all(l[~fin] == -np.inf)
    lse_err = float(np.abs(l[fin] - lse_ref[fin]).max()) if fin.any() else 0.0
    return float(err.max()), float(err.sum()), err.size, lse_err


def assert_attention_close(o_gpu: torch.Tensor, lse_gpu: torch.Tensor, O_ref: np.ndarray, lse_ref: np.ndarray, tag=None):
    mx, total, n, lse_err = attention_errors(o_gpu, lse_gpu, O_ref, lse_ref)
    if tag:
        record_maxima(tag, o_max=mx, o_mean=total / n, lse_max=lse_err)
    assert mx <= O_MAX_ABS, f"max-abs {mx}"
    assert total / n <= O_MEAN_ABS, f"mean-abs {total / n}"
    assert lse_err <= LSE_MAX_ABS, f"lse max-abs {lse_err}"
    return mx, total / n


# Gradients (bf16 outputs against the fp64 oracle).  The forward bars are stated for O, a convex combination of N(0,1)
# values.  A gradient element is a sum of products of either sign (dV_jc = sum_i p_ij dO_ic, ...), and what a bf16
# implementation gets wrong is relative to the PRODUCTS: p carries the forward's lse error (up to 0.7 %, the same
# sign for a whole row) and its own bf16 rounding, dS = p (dP - D) the rounding of O inside D.  So the bar per element
# is relative to the element's term magnitude M (oracle.masked_attention_bwd_magnitudes: the same sums with every
# product in absolute value), plus the output format's rounding of the element itself, plus a small floor:
#     |error| <= GRAD_TERM * M + 2^-8 * |reference| + GRAD_FLOOR,     mean |error| <= GRAD_TERM_MEAN * mean M.
# GRAD_TERM is about twice the largest ratio observed over the full-size workloads and the small cases (0.67 %; dV of
# the tiny random-block mask), GRAD_TERM_MEAN likewise (0.09 % observed).  Nothing in
# it depends on the tensor's overall size.  Where no magnitudes are at hand (rows and keys sampled out of heads that
# are not compared whole) the cruder form |error| <= 2e-2 * (1 + |reference|) is used.
GRAD_TERM, GRAD_TERM_MEAN, GRAD_OUT, GRAD_FLOOR = 1.5e-2, 2e-3, 2.0 ** -8, 1e-3
GRAD_ABS, GRAD_REL = O_MAX_ABS, 2e-2


def assert_grad_close(name: str, got_f64: np.ndarray, ref: np.ndarray, mag=None, tag=None):
    assert not np.isnan(got_f64).any(), name
    err = np.abs(got_f64 - ref)
    if mag is None:
        excess = err - GRAD_REL * np.abs(ref)
        if tag:
            record_maxima(f"{tag} {name}", max=err.max(), mean=err.mean(), ref_max=np.abs(ref).max(), abs_part_needed=max(0.0, float(excess.max())))
        assert excess.max() <= GRAD_ABS, f"{name}: an element is off by {excess.max():.3e} beyond {GRAD_REL} of its reference value"
        return err.max(), err.mean()
    assert mag.shape == ref.shape and np.all(mag >= np.abs(ref) - 1e-9)
    over = err - GRAD_OUT * np.abs(ref) - GRAD_FLOOR          # what the term-relative part has to cover
    ratio = float((over / np.maximum(mag, 1e-30)).max())
    mean_ratio = float(err.mean() / max(float(mag.mean()), 1e-30))
    if tag:
        record_maxima(f"{tag} {name}", max=err.max(), mean=err.mean(), ref_max=np.abs(ref).max(), mag_max=mag.max(), term_ratio=max(0.0, ratio),
                      mean_ratio=mean_ratio)
    assert ratio <= GRAD_TERM, f"{name}: an element is off by {ratio:.3e} of its term magnitude (max-abs error {err.max():.3e})"
    assert mean_ratio <= GRAD_TERM_MEAN, f"{name}: mean-abs error {err.mean():.3e} is {mean_ratio:.3e} of the mean term magnitude"
    return err.max(), err.mean()
