"""Brute-force companions used to pin the oracle.  Written separately from oracle/ on purpose:
they build the full L x L masked logit matrix (or sort every candidate) and lean on library
routines (scipy softmax / logsumexp, numpy argsort), so a mistake in the oracle's per-row
bookkeeping cannot be mirrored here."""
import numpy as np
from scipy.special import logsumexp, softmax


def dense_masked_attention(Q, K, V, mask, scale):
    """Q [Hq,Lq,D], K,V [Hkv,L,D], mask [Hq,Lq,L] bool (True = attend). fp64 outputs."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Hq, Hkv = Q.shape[0], K.shape[0]
    Kr = np.repeat(K, Hq // Hkv, axis=0)   # GQA: query head h reads kv head h // G
    Vr = np.repeat(V, Hq // Hkv, axis=0)
    logits = scale * np.einsum("hqd,htd->hqt", Q, Kr)
    logits = np.where(mask, logits, -np.inf)
    P = softmax(logits, axis=-1)
    return np.einsum("hqt,htd->hqd", P, Vr), logsumexp(logits, axis=-1), P


def causal_mask(Hq, Lq, L, q_pos0=0):
    i = (q_pos0 + np.arange(Lq))[:, None]
    t = np.arange(L)[None, :]
    return np.broadcast_to(t <= i, (Hq, Lq, L)).copy()


def span_mask(idx, S, L, q_pos0=0):
    """Mask of the attended set: selected spans below the query's own span + [c*S, i]."""
    Hq, Lq, k = idx.shape
    m = np.zeros((Hq, Lq, L), dtype=bool)
    for h in range(Hq):
        for r in range(Lq):
            i = q_pos0 + r
            c = i // S
            m[h, r, c * S:i + 1] = True
            for j in idx[h, r]:
                if 0 <= j < c:
                    m[h, r, j * S:(j + 1) * S] = True
    return m


def argsort_topk(scores, k):
    """Indices of the k largest entries, ties to the lower index, by a stable library sort."""
    scores = np.asarray(scores, dtype=np.float64)
    order = np.argsort(-scores, kind="stable")
    return np.sort(order[:k])


def gated_combination(Q, K, V, idx, scores, S, scale, q_pos0=0):
    """Algorithm 1's output rule by full masked matrices: one dense masked softmax per slot over
    (span of the slot) | (local window), library softmax over the slot scores, weighted sum.
    Rows without a valid slot get the window-only attention.  Q [Hq,Lq,D]; idx, scores [Hq,Lq,k]."""
    Q = np.asarray(Q, dtype=np.float64)
    Hq, Lq, _ = Q.shape
    L = K.shape[1]
    k = idx.shape[2]
    pos = q_pos0 + np.arange(Lq)
    c = pos // S
    t = np.arange(L)[None, None, :]
    window = (t >= (c * S)[None, :, None]) & (t <= pos[None, :, None])
    window = np.broadcast_to(window, (Hq, Lq, L))
    valid = (idx >= 0) & (idx < c[None, :, None])                       # [Hq,Lq,k]
    gate_logits = np.where(valid, np.asarray(scores, dtype=np.float64), -np.inf)
    any_valid = valid.any(axis=-1)
    alpha = np.zeros((Hq, Lq, k))
    alpha[any_valid] = softmax(gate_logits[any_valid], axis=-1)
    O = np.zeros(Q.shape)
    for n in range(k):
        j = idx[:, :, n]
        in_span = (t >= (j * S)[:, :, None]) & (t < ((j + 1) * S)[:, :, None]) & valid[:, :, n, None]
        A, _, _ = dense_masked_attention(Q, K, V, in_span | window, scale)
        O += alpha[:, :, n, None] * A
    Aw, _, _ = dense_masked_attention(Q, K, V, window, scale)
    O[~any_valid] = Aw[~any_valid]
    return O, alpha
