"""Dense numpy (float64) routines the CPU checker is pinned against.

Nothing here is shared with oracle/ or with the GPU library: attention is computed through
an explicit T x T boolean mask and whole-matrix softmax (the textbook form of Eq. 1 of the
paper with masked entries removed), gradients through the textbook matrix formulas, scores
through pooled dot products, selection through a full sort.
"""
import numpy as np


def nblocks(cu, B):
    return [(int(cu[s + 1] - cu[s]) + B - 1) // B for s in range(len(cu) - 1)]


def causal_same_sequence_mask(cu):
    """mask[r, c] = c is in r's sequence and c <= r (dense causal attention per sequence)."""
    T = int(cu[-1])
    seq = np.zeros(T, dtype=np.int64)
    for s in range(len(cu) - 1):
        seq[cu[s]:cu[s + 1]] = s
    r = np.arange(T)
    return (seq[:, None] == seq[None, :]) & (r[None, :] <= r[:, None])


def mask_from_selection(cu, B, NQB, rowptr, idx, hs):
    """Token-level mask of selection head hs built from the CSR block lists."""
    T = int(cu[-1])
    m = np.zeros((T, T), dtype=bool)
    nb = nblocks(cu, B)
    qb = 0
    for s in range(len(cu) - 1):
        L = int(cu[s + 1] - cu[s])
        for i in range(nb[s]):
            row = hs * NQB + qb + i
            r0, r1 = cu[s] + i * B, cu[s] + min((i + 1) * B, L)
            for j in idx[rowptr[row]:rowptr[row + 1]]:
                c0, c1 = cu[s] + j * B, cu[s] + min((j + 1) * B, L)
                m[r0:r1, c0:c1] = True
        qb += nb[s]
    m &= causal_same_sequence_mask(cu)
    return m


def masked_attention(Q, K, V, masks, scale):
    """Q [T,Hq,D]; K,V [T,Hkv,D]; masks: list of T x T bool, one per query head.
    Returns O [T,Hq,D], LSE [Hq,T], P list."""
    T, Hq, D = Q.shape
    G = Hq // K.shape[1]
    O = np.zeros((T, Hq, D))
    LSE = np.zeros((Hq, T))
    Ps = []
    for h in range(Hq):
        S = scale * (Q[:, h, :].astype(np.float64) @ K[:, h // G, :].astype(np.float64).T)
        S = np.where(masks[h], S, -np.inf)
        mx = S.max(axis=1, keepdims=True)
        E = np.exp(S - mx)
        l = E.sum(axis=1, keepdims=True)
        P = E / l
        O[:, h, :] = P @ V[:, h // G, :].astype(np.float64)
        LSE[h] = (mx + np.log(l))[:, 0]
        Ps.append(P)
    return O, LSE, Ps


def masked_attention_grads(Q, K, V, dO, masks, scale):
    """Matrix-form gradients of masked softmax attention."""
    T, Hq, D = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    O, _, Ps = masked_attention(Q, K, V, masks, scale)
    dQ = np.zeros((T, Hq, D)); dK = np.zeros((T, Hkv, D)); dV = np.zeros((T, Hkv, D))
    for h in range(Hq):
        g = h // G
        P = Ps[h]
        dOh = dO[:, h, :].astype(np.float64)
        dV[:, g, :] += P.T @ dOh
        dP = dOh @ V[:, g, :].astype(np.float64).T
        dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
        dQ[:, h, :] = scale * dS @ K[:, g, :].astype(np.float64)
        dK[:, g, :] += scale * dS.T @ Q[:, h, :].astype(np.float64)
    return dQ, dK, dV


def pooled_scores(cu, B, Q, K, score_scale, per_kvgroup):
    """Scores via <mean(Q block), mean(K block)> (summed over the group's heads if per_kvgroup).
    Returns a list over sequences of arrays [Hs, n, n] with -inf where j >= i."""
    Hq, Hkv = Q.shape[1], K.shape[1]
    G = Hq // Hkv
    out = []
    for s, n in enumerate(nblocks(cu, B)):
        L = int(cu[s + 1] - cu[s])
        qbar = np.zeros((n, Hq, Q.shape[2])); kbar = np.zeros((n, Hkv, Q.shape[2]))
        for j in range(n):
            sl = slice(cu[s] + j * B, cu[s] + min((j + 1) * B, L))
            qbar[j] = Q[sl].astype(np.float64).mean(axis=0)
            kbar[j] = K[sl].astype(np.float64).mean(axis=0)
        sc = np.einsum("ihd,jhd->hij", qbar, np.repeat(kbar, G, axis=1)) * score_scale
        if per_kvgroup:
            sc = sc.reshape(Hkv, G, n, n).sum(axis=1)
        ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
        sc[:, jj >= ii] = -np.inf
        out.append(sc)
    return out


def sort_select(row_scores, i, c):
    """Indices kept for query block i with c slots: diagonal + best c-1 of j<i, full sort."""
    cand = np.asarray(row_scores[:i], dtype=np.float32)
    key = np.where(np.isnan(cand), -np.inf, cand.astype(np.float64))
    nanflag = np.isnan(cand).astype(np.int64)           # NaN after every number, even -inf
    order = np.lexsort((np.arange(i), -key, nanflag))    # last key is primary
    return sorted(order[: c - 1].tolist()) + [i]
