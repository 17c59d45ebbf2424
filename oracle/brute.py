"""Oracle pins (test infrastructure): scalar-loop brute force for tiny inputs.

Independent second formulations used only to pin the vectorised oracle: attention iterates explicitly over
the allowed key set with math.exp / math.log; block counts use four nested loops over the zero-padded mask.
"""
import math
import numpy as np


def brute_attention(q, k, v, mask, scale):
    """q [B,H,N,d], k, v [B,H,Nk,d] float arrays; mask [Mb,N,Nk]; pure Python loops.  Returns (O, lse) as float64 arrays."""
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    O = np.zeros((B, H, N, d))
    lse = np.full((B, H, N), -math.inf)
    for b in range(B):
        mb = mask[b if Mb == B else 0]
        for h in range(H):
            for i in range(N):
                A = [j for j in range(k.shape[2]) if mb[i, j] != 0]
                if not A:
                    continue
                s = [scale * sum(float(q[b, h, i, c]) * float(k[b, h, j, c]) for c in range(d)) for j in A]
                mx = max(s)
                w = [math.exp(x - mx) for x in s]
                tot = sum(w)
                for c in range(d):
                    O[b, h, i, c] = sum(wj * float(v[b, h, j, c]) for wj, j in zip(w, A)) / tot
                lse[b, h, i] = mx + math.log(tot)
    return O, lse


def brute_block_counts(mask2d, Br, Bc):
    """Count of non-zero elements in every Br x Bc block of one N x Nk mask, zero-padded; 4 nested loops."""
    N, Nk = mask2d.shape
    nbr, nbc = -(-N // Br), -(-Nk // Bc)
    cnt = [[0] * nbc for _ in range(nbr)]
    for bi in range(nbr):
        for bj in range(nbc):
            c = 0
            for r in range(bi * Br, min(N, (bi + 1) * Br)):
                for s in range(bj * Bc, min(Nk, (bj + 1) * Bc)):
                    if mask2d[r, s] != 0:
                        c += 1
            cnt[bi][bj] = c
    return np.asarray(cnt, dtype=np.int64)


def brute_bwd_magnitudes(q, k, v, mask, do, scale):
    """Term magnitudes of the attention gradients (see attention_bwd.masked_attention_bwd_magnitudes), one (query, key)
    pair at a time in pure Python: p_ij from an explicit softmax over the allowed keys of row i, dP_ij and D_i from
    explicit dot products, every product added in absolute value (D_i enters as sum_c |dO_ic| |O_ic|).  q, k, v, do [B,H,N,d]; mask [Mb,N,N]."""
    B, H, N, d = q.shape
    Mb = mask.shape[0]
    MQ, MK, MV = np.zeros((B, H, N, d)), np.zeros((B, H, N, d)), np.zeros((B, H, N, d))
    for b in range(B):
        mb = mask[b if Mb == B else 0]
        for h in range(H):
            for i in range(N):
                A = [j for j in range(N) if mb[i, j] != 0]
                if not A:
                    continue
                s = [scale * sum(float(q[b, h, i, c]) * float(k[b, h, j, c]) for c in range(d)) for j in A]
                mx = max(s)
                w = [math.exp(x - mx) for x in s]
                tot = sum(w)
                p = [x / tot for x in w]
                dP = [sum(float(do[b, h, i, c]) * float(v[b, h, j, c]) for c in range(d)) for j in A]
                out = [sum(pj * float(v[b, h, j, c]) for pj, j in zip(p, A)) for c in range(d)]          # O_i
                d_abs = sum(abs(float(do[b, h, i, c])) * abs(out[c]) for c in range(d))
                for pj, dpj, j in zip(p, dP, A):
                    size = pj * (abs(dpj) + d_abs)
                    for c in range(d):
                        MV[b, h, j, c] += pj * abs(float(do[b, h, i, c]))
                        MQ[b, h, i, c] += scale * size * abs(float(k[b, h, j, c]))
                        MK[b, h, j, c] += scale * size * abs(float(q[b, h, i, c]))
    return MQ, MK, MV
