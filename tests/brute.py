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


def span_mask(idx, S, L, q_pos0=0, stride=None):
    """Mask of the attended set: selected spans below the query's own cell + the window [c*A, i].
    Anchors sit every A = stride tokens (default S); span j is the S tokens that end at its
    anchor (j+1)*A - 1, so with S > A the spans overlap and the mask is their union."""
    A = S if stride is None else stride
    Hq, Lq, k = idx.shape
    m = np.zeros((Hq, Lq, L), dtype=bool)
    for h in range(Hq):
        for r in range(Lq):
            i = q_pos0 + r
            c = i // A
            m[h, r, c * A:i + 1] = True
            for j in idx[h, r]:
                if 0 <= j < c:
                    m[h, r, max(0, (j + 1) * A - S):(j + 1) * A] = True
    return m


def argsort_topk(scores, k):
    """Indices of the k largest entries, ties to the lower index, by a stable library sort."""
    scores = np.asarray(scores, dtype=np.float64)
    order = np.argsort(-scores, kind="stable")
    return np.sort(order[:k])


def gated_combination(Q, K, V, idx, scores, S, scale, q_pos0=0, stride=None):
    """Algorithm 1's output rule by full masked matrices: one dense masked softmax per slot over
    (span of the slot) | (local window), library softmax over the slot scores, weighted sum.
    Rows without a valid slot get the window-only attention.  Q [Hq,Lq,D]; idx, scores [Hq,Lq,k]."""
    Q = np.asarray(Q, dtype=np.float64)
    Hq, Lq, _ = Q.shape
    L = K.shape[1]
    k = idx.shape[2]
    A_ = S if stride is None else stride
    pos = q_pos0 + np.arange(Lq)
    c = pos // A_
    t = np.arange(L)[None, None, :]
    window = (t >= (c * A_)[None, :, None]) & (t <= pos[None, :, None])
    window = np.broadcast_to(window, (Hq, Lq, L))
    valid = (idx >= 0) & (idx < c[None, :, None])                       # [Hq,Lq,k]
    gate_logits = np.where(valid, np.asarray(scores, dtype=np.float64), -np.inf)
    any_valid = valid.any(axis=-1)
    alpha = np.zeros((Hq, Lq, k))
    alpha[any_valid] = softmax(gate_logits[any_valid], axis=-1)
    O = np.zeros(Q.shape)
    for n in range(k):
        j = idx[:, :, n]
        in_span = (t >= ((j + 1) * A_ - S)[:, :, None]) & (t < ((j + 1) * A_)[:, :, None]) & valid[:, :, n, None]
        A, _, _ = dense_masked_attention(Q, K, V, in_span | window, scale)
        O += alpha[:, :, n, None] * A
    Aw, _, _ = dense_masked_attention(Q, K, V, window, scale)
    O[~any_valid] = Aw[~any_valid]
    return O, alpha


def check_selection_all_rows(idx, Qs, Ks, S, topk, q_pos0=0, margin=1e-3, chunk=16384):
    """Every row of a prefill span-search output against library routines, on the tensors' own device.

    idx [Hq, Lq, k] int32, Qs [Hq, Lq, D], Ks [Hkv, n, D] (torch tensors).  Per head and chunk of rows:
    the full score matrix by one fp64 matmul, the expected rows by a stable descending library sort
    (ties to the lower span index).  A row that differs from the expected one must (1) have its k-th
    and (k+1)-th scores within `margin`, (2) list min(k, c) distinct spans below c in ascending order,
    -1 padding last, (3) pick no span scoring more than `margin` below the k-th score and drop none
    scoring more than `margin` above it.  Returns (rows checked, rows that differ inside the margin);
    raises AssertionError on the first violation."""
    import torch

    Hq, Lq, k = idx.shape
    Hkv, n, _ = Ks.shape
    G = Hq // Hkv
    dev = idx.device
    ninf = float("-inf")
    span = torch.arange(n, device=dev)
    differ = 0
    for h in range(Hq):
        Kh = Ks[h // G].double()
        for r0 in range(0, Lq, chunk):
            r1 = min(Lq, r0 + chunk)
            c = (q_pos0 + torch.arange(r0, r1, device=dev)) // S                      # [R]
            sc = Qs[h, r0:r1].double() @ Kh.T                                          # [R, n]
            sc = torch.where(span[None, :] < c[:, None], sc, torch.full_like(sc, ninf))
            kk = torch.clamp(c, max=k)                                                 # spans to select
            order = torch.sort(sc, dim=1, descending=True, stable=True)
            kcols = min(k + 1, n)
            top_v, top_j = order.values[:, :kcols], order.indices[:, :kcols]
            if kcols < k + 1:
                pad = k + 1 - kcols
                top_v = torch.cat([top_v, torch.full((r1 - r0, pad), ninf, device=dev, dtype=top_v.dtype)], 1)
                top_j = torch.cat([top_j, torch.zeros((r1 - r0, pad), device=dev, dtype=top_j.dtype)], 1)
            slot = torch.arange(k, device=dev)[None, :]
            want = torch.where(slot < kk[:, None], top_j[:, :k], torch.full_like(top_j[:, :k], n + 1))
            want = torch.sort(want, dim=1).values
            want = torch.where(want > n, torch.full_like(want, -1), want)
            got = idx[h, r0:r1].long()
            valid = got >= 0
            # shape of every row
            assert torch.equal(valid.sum(1), kk), (h, r0, "number of listed spans")
            assert bool((valid[:, :-1] >= valid[:, 1:]).all()), (h, r0, "padding must come last")
            assert bool((got < c[:, None]).all()), (h, r0, "span at or beyond the query's own")
            both = valid[:, 1:] & valid[:, :-1]
            assert bool(((got[:, 1:] > got[:, :-1]) | ~both).all()), (h, r0, "ascending, distinct")
            bad = (got != want).any(1)
            nbad = int(bad.sum())
            if nbad == 0:
                continue
            differ += nbad
            rows = bad.nonzero()[:, 0]
            kb = kk[rows]
            assert bool((kb > 0).all())
            s_k = top_v[rows, kb - 1]
            s_k1 = top_v[rows, kb]                    # -inf when there is no (k+1)-th candidate
            assert bool((s_k - s_k1 < margin).all()), (h, r0, "a row outside the tie margin differs")
            scb, gotb, validb = sc[rows], got[rows], valid[rows]
            picked = torch.gather(scb, 1, gotb.clamp(min=0))
            picked = torch.where(validb, picked, torch.full_like(picked, float("inf")))
            assert bool((picked.min(1).values >= s_k - margin).all()), (h, r0, "picked a span below the margin")
            # scores of the spans that were not picked (empty slots point at a spare column)
            rest = torch.cat([scb, torch.full_like(scb[:, :1], ninf)], 1)
            rest.scatter_(1, torch.where(validb, gotb, torch.full_like(gotb, n)), ninf)
            assert bool((rest.max(1).values <= s_k + margin).all()), (h, r0, "dropped a span above the margin")
    return Hq * Lq, differ
