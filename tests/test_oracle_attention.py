"""Pins for oracle/attention.py: brute force, library routines, closed forms and invariants (CPU only)."""
import math
import numpy as np
import pytest
import torch

import oracle
from workloads import make_qkv, masks


def _rand_case(seed, B=2, H=2, N=24, d=8, Mb=1, p=0.4, empty_rows=(3, 17)):
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((B, H, N, d)) for _ in range(3))
    mask = (rng.random((Mb, N, N)) < p).astype(np.uint8)
    mask *= rng.integers(1, 255, size=mask.shape, dtype=np.uint8)     # any non-zero byte means "attend"
    for r in empty_rows:
        mask[:, r, :] = 0
    return q, k, v, mask


@pytest.mark.parametrize("Mb", [1, 2])
def test_matches_scalar_brute_force(Mb):
    q, k, v, mask = _rand_case(1, Mb=Mb)
    scale = 0.37
    O, lse = oracle.masked_attention(q, k, v, mask, scale=scale, row_chunk=7)
    Ob, lb = oracle.brute_attention(q, k, v, mask, scale)
    assert np.abs(O - Ob).max() < 1e-12
    fin = np.isfinite(lb)
    assert np.array_equal(np.isfinite(lse), fin)
    assert np.abs(lse[fin] - lb[fin]).max() < 1e-12
    assert not fin[:, :, 3].any() and not fin[:, :, 17].any()


def test_sampled_rows_match_full():
    q, k, v, mask = _rand_case(2, Mb=2)
    O, lse = oracle.masked_attention(q, k, v, mask)
    rows = [(0, 0, 0), (0, 1, 3), (1, 0, 17), (1, 1, 23), (1, 0, 5)]
    Or, lr = oracle.masked_attention_rows(q, k, v, mask, rows)
    for n, (b, h, i) in enumerate(rows):
        assert np.abs(Or[n] - O[b, h, i]).max() < 1e-13
        assert (lr[n] == lse[b, h, i]) or abs(lr[n] - lse[b, h, i]) < 1e-13


def test_fully_masked_rows_are_zero_and_no_nan():
    q, k, v, mask = _rand_case(3)
    O, lse = oracle.masked_attention(q, k, v, mask)
    assert not np.isnan(O).any() and not np.isnan(lse).any()
    assert np.all(O[:, :, 3] == 0) and np.all(lse[:, :, 3] == -np.inf)
    assert np.all(np.isfinite(lse[:, :, 4]))


def test_dense_mask_equals_library_attention():
    rng = np.random.default_rng(4)
    B, H, N, d = 2, 3, 40, 16
    q, k, v = (rng.standard_normal((B, H, N, d)) for _ in range(3))
    O, lse = oracle.masked_attention(q, k, v, masks.all_ones(N))
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy()
    assert np.abs(O - ref).max() < 1e-12
    s = torch.einsum("bhid,bhjd->bhij", tq, tk) / math.sqrt(d)
    assert np.abs(lse - torch.logsumexp(s, dim=-1).numpy()).max() < 1e-12


def test_causal_mask_equals_library_causal_attention():
    rng = np.random.default_rng(5)
    B, H, N, d = 1, 2, 33, 8
    q, k, v = (rng.standard_normal((B, H, N, d)) for _ in range(3))
    O, _ = oracle.masked_attention(q, k, v, masks.causal(N))
    ref = torch.nn.functional.scaled_dot_product_attention(*(torch.from_numpy(x) for x in (q, k, v)), is_causal=True).numpy()
    assert np.abs(O - ref).max() < 1e-12


def test_arbitrary_mask_equals_library_boolean_mask_attention():
    q, k, v, mask = _rand_case(6, empty_rows=())
    mask[:, np.arange(24), np.arange(24)] = 1          # no empty rows: the library has no convention for them
    ref = torch.nn.functional.scaled_dot_product_attention(
        *(torch.from_numpy(x) for x in (q, k, v)), attn_mask=torch.from_numpy(mask[0] != 0)).numpy()
    O, _ = oracle.masked_attention(q, k, v, mask)
    assert np.abs(O - ref).max() < 1e-12


def test_custom_scale_against_library():
    q, k, v, mask = _rand_case(7, empty_rows=())
    mask[:, np.arange(24), np.arange(24)] = 1
    ref = torch.nn.functional.scaled_dot_product_attention(
        *(torch.from_numpy(x) for x in (q, k, v)), attn_mask=torch.from_numpy(mask[0] != 0), scale=0.11).numpy()
    O, _ = oracle.masked_attention(q, k, v, mask, scale=0.11)
    assert np.abs(O - ref).max() < 1e-12


def test_zero_queries_give_mean_of_allowed_values_and_log_count():
    q, k, v, mask = _rand_case(8)
    q[:] = 0
    O, lse = oracle.masked_attention(q, k, v, mask)
    for b in range(2):
        for i in range(24):
            A = np.flatnonzero(mask[0, i])
            if A.size == 0:
                continue
            assert np.abs(O[b, :, i] - v[b][:, A].mean(axis=1)).max() < 1e-13
            assert np.abs(lse[b, :, i] - math.log(A.size)).max() < 1e-13


def test_single_allowed_key_returns_that_value_exactly():
    B, H, N, d = 1, 2, 32, 8
    qb, kb, vb = make_qkv(B, H, N, d, seed=9)
    perm = np.random.default_rng(9).permutation(N)
    mask = np.zeros((1, N, N), dtype=np.uint8)
    mask[0, np.arange(N), perm] = 1
    O, lse = oracle.masked_attention(qb, kb, vb, mask)
    vf, qf, kf = (oracle.bf16_bits_to_f64(x) for x in (vb, qb, kb))
    assert np.array_equal(O, vf[:, :, perm])
    s = np.einsum("bhid,bhid->bhi", qf, kf[:, :, perm]) / math.sqrt(d)
    assert np.abs(lse - s).max() < 1e-13


def test_joint_token_permutation_permutes_output():
    q, k, v, mask = _rand_case(10)
    pi = np.random.default_rng(10).permutation(24)
    O, lse = oracle.masked_attention(q, k, v, mask)
    Op, lp = oracle.masked_attention(q[:, :, pi], k[:, :, pi], v[:, :, pi], mask[:, pi][:, :, pi])
    assert np.abs(Op - O[:, :, pi]).max() < 1e-12
    fin = np.isfinite(lp)
    assert np.abs(lp[fin] - lse[:, :, pi][fin]).max() < 1e-12


def test_key_permutation_leaves_output_unchanged():
    q, k, v, mask = _rand_case(11)
    pi = np.random.default_rng(11).permutation(24)
    O, _ = oracle.masked_attention(q, k, v, mask)
    Op, _ = oracle.masked_attention(q, k[:, :, pi], v[:, :, pi], mask[:, :, pi])
    assert np.abs(Op - O).max() < 1e-12


def test_mask_is_per_batch_when_Mb_equals_B_and_shared_across_heads():
    q, k, v, mask = _rand_case(12, Mb=2)
    O, _ = oracle.masked_attention(q, k, v, mask)
    for b in range(2):
        Ob, _ = oracle.masked_attention(q[b:b + 1], k[b:b + 1], v[b:b + 1], mask[b:b + 1])
        assert np.array_equal(O[b], Ob[0])
    # heads see the same mask: swapping heads of the inputs swaps the outputs
    Os, _ = oracle.masked_attention(q[:, ::-1], k[:, ::-1], v[:, ::-1], mask)
    assert np.array_equal(Os, O[:, ::-1])


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x3DCD, 0x7F7F], dtype=np.uint16)
    want = [1.0, -1.0, 3.140625, 0.0, -0.0, 0.10009765625, 3.3895313892515355e38]
    got = oracle.bf16_bits_to_f64(bits)
    assert np.array_equal(got, np.array(want))
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, t)


def test_softmax_weights_sum_to_one_and_lse_shift():
    """Adding a constant c to every allowed score (K -> K + c*u where q.u = 1) shifts lse by scale*c and leaves O."""
    q, k, v, mask = _rand_case(13)
    O, lse = oracle.masked_attention(q, k, v, mask, scale=1.0)
    q2 = q.copy(); q2[..., 0] = 1.0
    k2 = k.copy(); k3 = k.copy(); k3[..., 0] += 2.5
    O2, l2 = oracle.masked_attention(q2, k2, v, mask, scale=1.0)
    O3, l3 = oracle.masked_attention(q2, k3, v, mask, scale=1.0)
    fin = np.isfinite(l2)
    assert np.abs(O3 - O2).max() < 1e-12
    assert np.abs(l3[fin] - l2[fin] - 2.5).max() < 1e-12


def test_rectangular_mask_new_queries_against_a_longer_key_cache():
    """Nq != Nk: brute force, the library routine, and "the last Nq rows of the square problem"."""
    rng = np.random.default_rng(14)
    B, H, Nq, Nk, d = 2, 2, 7, 19, 8
    q = rng.standard_normal((B, H, Nq, d))
    k, v = (rng.standard_normal((B, H, Nk, d)) for _ in range(2))
    mask = (rng.random((2, Nq, Nk)) < 0.5).astype(np.uint8)
    mask[:, 3] = 0
    O, lse = oracle.masked_attention(q, k, v, mask, scale=0.3, row_chunk=4)
    Ob, lb = oracle.brute_attention(q, k, v, mask, 0.3)
    fin = np.isfinite(lb)
    assert O.shape == (B, H, Nq, d) and np.abs(O - Ob).max() < 1e-12 and np.array_equal(np.isfinite(lse), fin)
    assert np.abs(lse[fin] - lb[fin]).max() < 1e-12 and not fin[:, :, 3].any()
    rows = [(0, 0, 0), (1, 1, 6), (1, 0, 3)]
    Or, lr = oracle.masked_attention_rows(q, k, v, mask, rows)
    O2, l2 = oracle.masked_attention(q, k, v, mask)
    for n, (b, h, i) in enumerate(rows):
        assert np.abs(Or[n] - O2[b, h, i]).max() < 1e-13
    mask[:, 3, 0] = 1
    ref = torch.nn.functional.scaled_dot_product_attention(
        *(torch.from_numpy(x) for x in (q, k, v)), attn_mask=torch.from_numpy(mask != 0)[:, None], scale=0.3).numpy()
    assert np.abs(oracle.masked_attention(q, k, v, mask, scale=0.3)[0] - ref).max() < 1e-12
    # the new tokens are the last Nq rows of a square problem over all Nk tokens
    qs = rng.standard_normal((B, H, Nk, d))
    sq = (rng.random((2, Nk, Nk)) < 0.5).astype(np.uint8)
    Os, ls = oracle.masked_attention(qs, k, v, sq)
    Ot, lt = oracle.masked_attention(qs[:, :, -Nq:], k, v, sq[:, -Nq:])
    assert np.array_equal(Ot, Os[:, :, -Nq:]) and np.array_equal(lt, ls[:, :, -Nq:])
