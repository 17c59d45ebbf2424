"""Pins for oracle/attention_bwd.py: finite differences of the (separately pinned) forward oracle, the library's
automatic differentiation of a dense masked softmax, closed forms and invariants (CPU only)."""
import math
import numpy as np
import pytest
import torch

import oracle
from workloads import masks
from test_oracle_attention import _rand_case


def _loss(q, k, v, mask, do, scale):
    O, _ = oracle.masked_attention(q, k, v, mask, scale=scale)
    return float((O * do).sum())


@pytest.mark.parametrize("Mb", [1, 2])
def test_matches_central_differences_of_the_forward_oracle(Mb):
    """L = sum(O * dO) with O from oracle.masked_attention; dL/dx by central differences at sampled coordinates."""
    q, k, v, mask = _rand_case(21, B=2, H=2, N=12, d=4, Mb=Mb, empty_rows=(5,))
    rng = np.random.default_rng(22)
    do = rng.standard_normal(q.shape)
    scale = 0.43
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do, scale=scale, row_chunk=5)
    eps = 1e-6
    for grad, which in ((dQ, 0), (dK, 1), (dV, 2)):
        for _ in range(40):
            pos = tuple(int(rng.integers(s)) for s in q.shape)
            args = [q.copy(), k.copy(), v.copy()]
            args[which][pos] += eps
            up = _loss(*args, mask, do, scale)
            args[which][pos] -= 2 * eps
            dn = _loss(*args, mask, do, scale)
            assert abs((up - dn) / (2 * eps) - grad[pos]) < 1e-7, (which, pos)


def test_matches_library_autograd_on_a_dense_masked_softmax():
    q, k, v, mask = _rand_case(23, B=2, H=3, N=24, d=8, Mb=2, empty_rows=())
    mask[:, np.arange(24), np.arange(24)] = 1
    do = np.random.default_rng(24).standard_normal(q.shape)
    tq, tk, tv = (torch.from_numpy(x).requires_grad_() for x in (q, k, v))
    allowed = torch.from_numpy(mask != 0)[:, None]                      # [Mb,1,N,N]: one mask for all heads
    O = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=allowed, scale=0.21)
    O.backward(torch.from_numpy(do))
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do, scale=0.21)
    for got, want in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        assert np.abs(got - want.numpy()).max() < 1e-12


def test_causal_mask_against_library_autograd():
    rng = np.random.default_rng(25)
    B, H, N, d = 1, 2, 33, 8
    q, k, v, do = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    tq, tk, tv = (torch.from_numpy(x).requires_grad_() for x in (q, k, v))
    torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).backward(torch.from_numpy(do))
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, masks.causal(N), do)
    for got, want in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        assert np.abs(got - want.numpy()).max() < 1e-12


def test_fully_masked_rows_and_unattended_keys_get_zero_gradient():
    q, k, v, mask = _rand_case(26, empty_rows=(3, 17))
    mask[:, :, 7] = 0                                                    # nobody attends key 7
    do = np.random.default_rng(27).standard_normal(q.shape)
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do)
    assert not any(np.isnan(x).any() for x in (dQ, dK, dV))
    assert np.all(dQ[:, :, 3] == 0) and np.all(dQ[:, :, 17] == 0)
    assert np.all(dK[:, :, 7] == 0) and np.all(dV[:, :, 7] == 0)
    # the upstream gradient of a fully masked row is irrelevant
    do2 = do.copy()
    do2[:, :, 3] = 100.0
    for a, b in zip((dQ, dK, dV), oracle.masked_attention_bwd(q, k, v, mask, do2)):
        assert np.array_equal(a, b)


def test_single_allowed_key_routes_dO_to_dV_and_nothing_to_dQ_dK():
    """One allowed key per row: p = 1 there, so dV_j = sum of dO over the rows that chose j, dS = 0."""
    rng = np.random.default_rng(28)
    B, H, N, d = 1, 2, 16, 4
    q, k, v, do = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    choice = rng.integers(0, N, size=N)
    mask = np.zeros((1, N, N), dtype=np.uint8)
    mask[0, np.arange(N), choice] = 1
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do)
    want = np.zeros_like(v)
    for i, j in enumerate(choice):
        want[:, :, j] += do[:, :, i]
    assert np.abs(dV - want).max() < 1e-13
    assert np.abs(dQ).max() < 1e-13 and np.abs(dK).max() < 1e-13


def test_zero_queries_closed_form():
    """q = 0: p is uniform over A_i, so dV_j = sum_{i: j in A_i} dO_i / |A_i| and dK = 0; dQ_i is scale times the
    p-weighted covariance of <dO_i, v_j> and k_j over A_i."""
    q, k, v, mask = _rand_case(29, B=1, H=2, N=24, d=8)
    q[:] = 0
    do = np.random.default_rng(30).standard_normal(q.shape)
    scale = 0.3
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do, scale=scale)
    assert np.abs(dK).max() < 1e-13
    wantV = np.zeros_like(v)
    for i in range(24):
        A = np.flatnonzero(mask[0, i])
        if A.size == 0:
            continue
        wantV[:, :, A] += do[:, :, i:i + 1] / A.size
        for h in range(2):
            g = v[0, h, A] @ do[0, h, i]
            cov = ((g - g.mean())[:, None] * k[0, h, A]).mean(axis=0)
            assert np.abs(dQ[0, h, i] - scale * cov).max() < 1e-13
    assert np.abs(dV - wantV).max() < 1e-13


def test_dS_rows_sum_to_zero_so_a_common_key_offset_leaves_dQ_unchanged_and_dK_sums_to_zero():
    q, k, v, mask = _rand_case(31)
    do = np.random.default_rng(32).standard_normal(q.shape)
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do, scale=1.0)
    # softmax is invariant to adding u to every key, so L is too: sum_j dK_j = 0
    assert np.abs(dK.sum(axis=2)).max() < 1e-12
    u = np.random.default_rng(33).standard_normal(8)
    dQ2, dK2, dV2 = oracle.masked_attention_bwd(q, k + u, v, mask, do, scale=1.0)
    assert np.abs(dQ2 - dQ).max() < 1e-11 and np.abs(dK2 - dK).max() < 1e-11 and np.abs(dV2 - dV).max() < 1e-11


def test_joint_token_permutation_permutes_gradients():
    q, k, v, mask = _rand_case(34)
    do = np.random.default_rng(35).standard_normal(q.shape)
    pi = np.random.default_rng(36).permutation(24)
    g = oracle.masked_attention_bwd(q, k, v, mask, do)
    gp = oracle.masked_attention_bwd(q[:, :, pi], k[:, :, pi], v[:, :, pi], mask[:, pi][:, :, pi], do[:, :, pi])
    for a, b in zip(g, gp):
        assert np.abs(b - a[:, :, pi]).max() < 1e-12


def test_sampled_rows_and_columns_match_full():
    q, k, v, mask = _rand_case(37, Mb=2)
    do = np.random.default_rng(38).standard_normal(q.shape)
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, mask, do, scale=0.2)
    picks = [(0, 0, 0), (0, 1, 3), (1, 0, 17), (1, 1, 23), (1, 0, 5)]
    r = oracle.masked_attention_bwd_rows(q, k, v, mask, do, picks, scale=0.2)
    ck, cv = oracle.masked_attention_bwd_cols(q, k, v, mask, do, picks, scale=0.2)
    for n, (b, h, i) in enumerate(picks):
        assert np.abs(r[n] - dQ[b, h, i]).max() < 1e-13
        assert np.abs(ck[n] - dK[b, h, i]).max() < 1e-13
        assert np.abs(cv[n] - dV[b, h, i]).max() < 1e-13


def test_bf16_bit_inputs_are_widened_exactly():
    from workloads import make_qkv
    qb, kb, vb = make_qkv(1, 2, 16, 8, seed=39)
    dob = make_qkv(1, 2, 16, 8, seed=40)[0]
    mask = masks.causal(16)
    a = oracle.masked_attention_bwd(qb, kb, vb, mask, dob)
    b = oracle.masked_attention_bwd(*(oracle.bf16_bits_to_f64(x) for x in (qb, kb, vb)), mask, oracle.bf16_bits_to_f64(dob))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_hand_worked_two_by_two():
    """N = 2, d = 1, scale = 1, q = 0 (uniform p = 1/2), k = (2, 5), v = (1, 3), dO = (1, 1), all pairs allowed:
    O = 2; dV_j = 1/2 + 1/2 = 1; dP_i = (1, 3), D_i = 2, dS_i = (-1/2, +1/2); dQ_i = -1/2*2 + 1/2*5 = 3/2; dK = 0."""
    q = np.zeros((1, 1, 2, 1))
    k = np.array([2.0, 5.0]).reshape(1, 1, 2, 1)
    v = np.array([1.0, 3.0]).reshape(1, 1, 2, 1)
    do = np.ones((1, 1, 2, 1))
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, np.ones((1, 2, 2), dtype=np.uint8), do, scale=1.0)
    assert np.allclose(dQ.ravel(), [1.5, 1.5], atol=1e-15) and np.allclose(dK.ravel(), [0, 0], atol=1e-15)
    assert np.allclose(dV.ravel(), [1.0, 1.0], atol=1e-15)
    # mask out key 1 for query 0: its row sees one key only (p = 1, dS = 0, dQ_0 = 0); dV_0 = 1 + 1/2, dV_1 = 1/2
    m = np.array([[[1, 0], [1, 1]]], dtype=np.uint8)
    dQ, dK, dV = oracle.masked_attention_bwd(q, k, v, m, do, scale=1.0)
    assert np.allclose(dQ.ravel(), [0.0, 1.5], atol=1e-15) and np.allclose(dV.ravel(), [1.5, 0.5], atol=1e-15)


def test_term_magnitudes_against_pair_by_pair_loops_and_the_triangle_inequality():
    """The yardstick of the gradient tolerances: equal to the scalar-loop formulation, never below the absolute value of
    the gradient it belongs to, equal to it where every term has one sign (dV with dO >= 0), and zero exactly where the
    gradient has no terms (fully masked query rows, keys nobody attends)."""
    q, k, v, mask = _rand_case(61, B=2, H=2, N=11, d=3, Mb=2, empty_rows=(4,))
    mask[:, :, 7] = 0                                              # a key nobody attends
    do = np.random.default_rng(62).standard_normal(q.shape)
    scale = 0.37
    got = oracle.masked_attention_bwd_magnitudes(q, k, v, mask, do, scale=scale, row_chunk=4)
    want = oracle.brute_bwd_magnitudes(q, k, v, mask, do, scale)
    grads = oracle.masked_attention_bwd(q, k, v, mask, do, scale=scale)
    for g, w, gr in zip(got, want, grads):
        assert np.abs(g - w).max() < 1e-12
        assert np.all(g >= np.abs(gr) - 1e-12)
    assert np.all(got[0][:, :, 4] == 0) and np.all(got[1][:, :, 7] == 0) and np.all(got[2][:, :, 7] == 0)
    pos = np.abs(do)
    MV = oracle.masked_attention_bwd_magnitudes(q, k, v, mask, pos, scale=scale)[2]
    assert np.abs(MV - oracle.masked_attention_bwd(q, k, v, mask, pos, scale=scale)[2]).max() < 1e-12
