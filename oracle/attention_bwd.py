"""Oracle (test infrastructure): gradients of masked softmax attention, written out from the definition, in fp64.

The paper times forward plus backward (Sec. 5 "Evaluation Metrics"; Appendix "Forward and Backward Pass
Performance Comparisons") and relies on Flash Attention's backward, which recomputes the attention matrix
(Sec. 3 "Flash Attention"); it prints no backward formulas.  The method stays exact, so the expected result is
the derivative of the forward definition of Sec. 3 "Standard Attention" restricted to the allowed keys.  With

    s_ij = scale * <q_i, k_j>,  A_i = { j : mask[i, j] != 0 },  p_ij = softmax_{A_i}(s_i)_j  (0 outside A_i),
    O_i = sum_j p_ij v_j,  and an upstream gradient dO (the loss is any L with dL/dO = dO),

the chain rule through the row-wise softmax gives

    dV_j = sum_i p_ij dO_i
    dP_ij = <dO_i, v_j>,   D_i = sum_j p_ij dP_ij  (= <dO_i, O_i>)
    dS_ij = p_ij (dP_ij - D_i)
    dQ_i = scale * sum_j dS_ij k_j,      dK_j = scale * sum_i dS_ij q_i.

Readings where the paper is silent: a query row with A_i empty has O_i = 0 whatever the inputs, so it contributes
nothing to any gradient and its dQ is 0; the mask has Mb = 1 or B planes and is shared by the heads.
"""
import numpy as np

from .attention import _as_f64


def _row_softmax(s, allowed):
    """Row-wise softmax over the allowed entries; rows without any allowed entry give all zeros."""
    s = np.where(allowed, s, -np.inf)
    has = allowed.any(axis=1)
    m = np.where(has, s.max(axis=1, initial=-np.inf), 0.0)
    p = np.exp(s - m[:, None])
    l = p.sum(axis=1)
    return p / np.where(has, l, 1.0)[:, None]


def masked_attention_bwd(q, k, v, mask, do, scale=None, row_chunk=512):
    """q, k, v, do: [B,H,N,d] (uint16 bf16 bit patterns or float arrays); mask [Mb,N,N], non-zero = attend.

    Returns dQ, dK, dV float64 [B,H,N,d] for the upstream gradient do."""
    q, k, v, do = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(do)
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    assert mask.shape == (Mb, N, N) and Mb in (1, B) and do.shape == q.shape
    scale = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    dQ, dK, dV = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b in range(B):
        mb = mask[b if Mb == B else 0]
        for r0 in range(0, N, row_chunk):
            r1 = min(N, r0 + row_chunk)
            allowed = mb[r0:r1] != 0
            for h in range(H):
                p = _row_softmax(scale * (q[b, h, r0:r1] @ k[b, h].T), allowed)      # [R, N]
                dV[b, h] += p.T @ do[b, h, r0:r1]
                dP = do[b, h, r0:r1] @ v[b, h].T                                      # [R, N]
                D = (p * dP).sum(axis=1)
                dS = p * (dP - D[:, None])
                dQ[b, h, r0:r1] = scale * (dS @ k[b, h])
                dK[b, h] += scale * (dS.T @ q[b, h, r0:r1])
    return dQ, dK, dV


def masked_attention_bwd_magnitudes(q, k, v, mask, do, scale=None, row_chunk=512):
    """Size of the terms each gradient element is a sum of (not a gradient: the yardstick against which the rounding
    error of a reduced-precision implementation of masked_attention_bwd is judged).  Every element of dV, dQ, dK above is a
    sum of products of either sign; an implementation that carries a relative error eps in p_ij, dP_ij or the terms of
    D_i is off by about eps times the sum of the ABSOLUTE values of those products, however small the element itself
    comes out:

        MV_jc = sum_i p_ij |dO_ic|
        MQ_ic = scale * sum_j p_ij (|dP_ij| + Dabs_i) |k_jc|,      Dabs_i = sum_c |dO_ic| |O_ic|
        MK_jc = scale * sum_i p_ij (|dP_ij| + Dabs_i) |q_ic|

    (dS_ij = p_ij (dP_ij - D_i) is itself a difference, and D_i = <dO_i, O_i> a sum of either sign formed from an output
    O that an implementation holds in rounded form; hence |dP| + Dabs.)  By the triangle inequality each magnitude
    bounds the absolute value of its gradient element.  Same arguments and shapes as masked_attention_bwd."""
    q, k, v, do = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(do)
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    assert mask.shape == (Mb, N, N) and Mb in (1, B) and do.shape == q.shape
    scale = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    MQ, MK, MV = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b in range(B):
        mb = mask[b if Mb == B else 0]
        for r0 in range(0, N, row_chunk):
            r1 = min(N, r0 + row_chunk)
            allowed = mb[r0:r1] != 0
            for h in range(H):
                p = _row_softmax(scale * (q[b, h, r0:r1] @ k[b, h].T), allowed)
                MV[b, h] += p.T @ np.abs(do[b, h, r0:r1])
                dP = do[b, h, r0:r1] @ v[b, h].T
                Dabs = (np.abs(do[b, h, r0:r1]) * np.abs(p @ v[b, h])).sum(axis=1)
                w = p * (np.abs(dP) + Dabs[:, None])
                MQ[b, h, r0:r1] = scale * (w @ np.abs(k[b, h]))
                MK[b, h] += scale * (w.T @ np.abs(q[b, h, r0:r1]))
    return MQ, MK, MV


def masked_attention_bwd_rows(q, k, v, mask, do, rows, scale=None):
    """dQ of sampled query rows (b, h, i), each from its own row of the definition alone.  Returns [len(rows), d]."""
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    scale = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    out = np.zeros((len(rows), d), dtype=np.float64)
    cache = {}
    for n, (b, h, i) in enumerate(rows):
        if (b, h) not in cache:
            cache.clear()
            cache[(b, h)] = (_as_f64(k[b, h]), _as_f64(v[b, h]))
        kk, vv = cache[(b, h)]
        idx = np.flatnonzero(mask[b if Mb == B else 0, i])
        if idx.size == 0:
            continue
        s = scale * (kk[idx] @ _as_f64(q[b, h, i]))
        p = np.exp(s - s.max())
        p /= p.sum()
        dP = vv[idx] @ _as_f64(do[b, h, i])
        dS = p * (dP - p @ dP)
        out[n] = scale * (dS @ kk[idx])
    return out


def masked_attention_bwd_cols(q, k, v, mask, do, cols, scale=None):
    """dK and dV of sampled key rows (b, h, j): sums over the queries i that may attend key j, each evaluated from its
    own row of the definition (softmax over A_i only).  Returns (dK [len(cols), d], dV [len(cols), d])."""
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    scale = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    dK = np.zeros((len(cols), d), dtype=np.float64)
    dV = np.zeros((len(cols), d), dtype=np.float64)
    for n, (b, h, j) in enumerate(cols):
        mb = mask[b if Mb == B else 0]
        kk, vv = _as_f64(k[b, h]), _as_f64(v[b, h])
        for i in np.flatnonzero(mb[:, j]):
            idx = np.flatnonzero(mb[i])
            at = int(np.searchsorted(idx, j))                       # position of key j among the allowed keys of row i
            qi, di = _as_f64(q[b, h, i]), _as_f64(do[b, h, i])
            s = scale * (kk[idx] @ qi)
            p = np.exp(s - s.max())
            p /= p.sum()
            dP = vv[idx] @ di
            dV[n] += p[at] * di
            dK[n] += scale * p[at] * (dP[at] - p @ dP) * qi
    return dK, dV
