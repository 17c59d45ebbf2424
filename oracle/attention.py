"""Oracle (test infrastructure): masked softmax attention written out as its definition, in fp64.

The method is exact (paper Sec. 2: unlike block-sparse approximations it computes exact attention; Sec. 4:
a skipped block has only masked elements, and inside the all-ones run no element is masked), so the
expected result is the plain definition of Sec. 3 "Standard Attention" restricted to the allowed keys:

    s_ij = scale * <q_i, k_j>,   A_i = { j : mask[i, j] != 0 }
    O_i  = sum_{j in A_i} softmax_{A_i}(s_i)_j * v_j,     lse_i = log sum_{j in A_i} exp(s_ij)

Readings where the paper is silent: scale is an argument (1/sqrt(d) by default); a row with A_i empty gives
O_i = 0 and lse_i = -inf; the mask has Mb = 1 (shared by the batch) or Mb = B planes and is always shared by
the heads (Sec. 1, insight (2)).  Queries and keys may differ in number (a block of new tokens attending a longer
key/value cache, as when a candidate tree is verified against its prefix, Sec. 5): q is [B,H,Nq,d], k and v are
[B,H,Nk,d], the mask [Mb,Nq,Nk]; the definition does not change.
"""
import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _as_f64(x):
    return bf16_bits_to_f64(x) if x.dtype == np.uint16 else np.asarray(x, dtype=np.float64)


def masked_attention(q, k, v, mask, scale=None, row_chunk=512):
    """q: [B,H,N,d], k, v: [B,H,Nk,d] (uint16 bf16 bit patterns or float arrays); mask: [Mb,N,Nk], non-zero = attend.

    Returns O float64 [B,H,N,d] and lse float64 [B,H,N] (natural log; -inf on fully masked rows)."""
    q, k, v = _as_f64(q), _as_f64(k), _as_f64(v)
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    assert k.shape == v.shape == (B, H, k.shape[2], d) and mask.shape == (Mb, N, k.shape[2]) and Mb in (1, B)
    scale = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    O = np.zeros((B, H, N, d), dtype=np.float64)
    lse = np.full((B, H, N), -np.inf, dtype=np.float64)
    for b in range(B):
        mb = mask[b if Mb == B else 0]
        for r0 in range(0, N, row_chunk):
            r1 = min(N, r0 + row_chunk)
            allowed = mb[r0:r1] != 0                                  # [R, N]
            has_key = allowed.any(axis=1)                             # [R]
            for h in range(H):
                s = scale * (q[b, h, r0:r1] @ k[b, h].T)              # [R, N]
                s = np.where(allowed, s, -np.inf)
                m = np.where(has_key, s.max(axis=1, initial=-np.inf), 0.0)
                p = np.exp(s - m[:, None])                            # exp(-inf) = 0 on masked elements
                l = p.sum(axis=1)
                with np.errstate(divide="ignore", invalid="ignore"):
                    o = (p @ v[b, h]) / l[:, None]
                    ls = m + np.log(l)
                O[b, h, r0:r1] = np.where(has_key[:, None], o, 0.0)
                lse[b, h, r0:r1] = np.where(has_key, ls, -np.inf)
    return O, lse


def masked_attention_rows(q, k, v, mask, rows, scale=None):
    """The same definition evaluated one query row at a time for sampled (b, h, i) triples.

    Returns O float64 [len(rows), d] and lse float64 [len(rows)].  Used at sizes where the full N x N
    score matrix per head is too slow to form."""
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    scale = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    O = np.zeros((len(rows), d), dtype=np.float64)
    lse = np.full(len(rows), -np.inf, dtype=np.float64)
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
        m = s.max()
        p = np.exp(s - m)
        l = p.sum()
        O[n] = (p @ vv[idx]) / l
        lse[n] = m + np.log(l)
    return O, lse
