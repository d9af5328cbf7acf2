"""CPU fp64 oracle for the N=2 Superlinear attention hot path (span-search + span-attention).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: it is called
by the tests, by the smoke check and by the benchmark's cpu-baseline leg.  It shares no code
with the HIP kernels and never reads their output.

What it computes is the *definition* of the result, written out per query row in float64:

* span-search  -- Section 3.2, eq. (2) (score = <Q_s(i), K_a(t)>) and eq. (3) (TopK over the
  candidate anchors), with the candidate set of Algorithm 1 (anchors minus the local window).
* span-attention -- Section 3.3, eq. (4): standard scaled dot-product attention over the keys
  of the selected spans, merged (de-duplicated) with the local window as in Algorithm 1
  (the DedupConcat step).  The empty-selection branch of Algorithm 1 (attend the window only)
  falls out of the same code.

Geometry (fixed span grid).  The span grid specialises the paper's span construction
(Section 3.3, Algorithm 1: S_t = [t - b*l, t + f*l]) to f = 0 and b*l = S for every query:
span j is the token range [j*S, (j+1)*S - 1] and its anchor is its last token
t_j = (j+1)*S - 1.  The query at absolute position i lies in span c = i // S; its local
window W is [c*S, i]; its candidate anchors are the spans j < c (window indices are excluded
from the candidates, Algorithm 1).  K_a = K (Section 3.5 / 4.2), so the default search key of
span j is K[t_j].

Redundant grid (Section 2.4: p_sh + p_sp > 1; Section 4.4's redundancy factors): anchors every
`stride` tokens with spans S > stride tokens long, so that neighbouring spans overlap; the
attended set is then the set UNION of the selected spans and the window (DedupConcat), and the
search runs on the anchor grid (S = stride in the search functions).

Readings of points the paper leaves open (all listed in the design notes of the repository):
ties in TopK go to the lower span index; selected spans are reported in ascending index order
and padded with -1; selection is per query head; the search score is the raw dot product (no
scale); attention uses one joint softmax over the union of the selected spans and the local
window, scale 1/sqrt(D) unless given; LSE is the natural-log sum of exp(logit) over that set.

* combination -- Section 3.4, eq. (5)-(6), and Algorithm 1's last steps: per selected span t the
  attention A_t over J_t = DedupConcat(S_t, W) with its own softmax, then
  O = sum_t alpha_t A_t with alpha = softmax of the search scores of the selected spans; with
  nothing selected, attention over the window alone.  (The joint softmax above is what the
  task statement fixes for span-attention; the gate is the paper's own output rule.)

* the paper's own geometry -- Section 3.3 with Fig. 3, Algorithm 1, for p = 1/root (root = 2, or
  3 for the (1/3, 2/3) exponent split of Section 5): anchors t_s = i - (s+1)^root + 1, base span
  length l(i) = ceil(i^(1-p)) in exact integer arithmetic, spans [t - b*l, min(i, t + f*l)],
  window [i - w + 1, i] whose indices are removed from the candidates; search, span-attention
  and combination per query row (anchor_* functions).  Ties go to the nearer anchor.

Every function is pinned by tests that do not call it back: brute-force dense causal
attention, brute-force argsort, closed forms, a library softmax with an explicit mask, the
values the paper prints for its worked example and hand-derived values stored under
tests/golden/.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


def _f64(a):
    """Widen anything array-like (numpy, or an object exposing .numpy()) to float64."""
    return np.asarray(a, dtype=F64)


def n_spans(L: int, S: int) -> int:
    """Number of grid spans touching [0, L): ceil(L / S)."""
    return -(-int(L) // int(S))


def anchor_of_span(j: int, S: int) -> int:
    """Anchor token of span j: its last token (Algorithm 1's span with f = 0 ends at the anchor)."""
    return (int(j) + 1) * int(S) - 1


def span_keys(K, S: int):
    """Search keys K_a(t_j) = K[t_j] for every *complete* span j (Section 3.5: K_a = K).

    K: [Hkv, L, D].  Returns [Hkv, L // S, D] float64.
    """
    K = np.asarray(K)
    L = K.shape[1]
    nfull = L // S
    anchors = [anchor_of_span(j, S) for j in range(nfull)]
    return _f64(K[:, anchors, :])


def search_scores_row(qs, Ks_kv, c: int):
    """Eq. (2): s_j = sum_d Qs[d] * Ks[j, d] for the candidate spans j = 0 .. c-1 (no scale)."""
    if c <= 0:
        return np.zeros((0,), dtype=F64)
    return _f64(Ks_kv[:c]) @ _f64(qs)


def select_topk(scores, k: int):
    """Eq. (3) with the tie rule: the min(k, len) largest scores, ties to the lower index.

    Returns the selected indices in ascending index order (a python list of ints).
    """
    scores = _f64(scores)
    order = sorted(range(scores.shape[0]), key=lambda j: (-scores[j], j))
    return sorted(order[: max(0, int(k))])


def span_search(Qs, Ks, S: int, topk: int, q_pos0: int = 0, return_scores: bool = False):
    """Span-search for every (head, query row).

    Qs: [Hq, Lq, D] search queries; Ks: [Hkv, n, D] span search keys (n >= number of complete
    spans below the last query); query row r sits at absolute position q_pos0 + r.
    Returns idx [Hq, Lq, topk] int32 (ascending span indices, -1 padding) and, if asked, the
    fp64 scores of the selected spans in the same slots (-inf in padded slots).
    """
    Qs = np.asarray(Qs)
    Ks = np.asarray(Ks)
    Hq, Lq, _ = Qs.shape
    Hkv = Ks.shape[0]
    G = Hq // Hkv
    idx = np.full((Hq, Lq, topk), -1, dtype=np.int32)
    sc = np.full((Hq, Lq, topk), -np.inf, dtype=F64)
    for h in range(Hq):
        kv = h // G
        for r in range(Lq):
            i = q_pos0 + r
            c = i // S
            s = search_scores_row(Qs[h, r], Ks[kv], c)
            sel = select_topk(s, topk)
            for slot, j in enumerate(sel):
                idx[h, r, slot] = j
                sc[h, r, slot] = s[j]
    if return_scores:
        return idx, sc
    return idx


def selection_margin(scores, k: int) -> float:
    """Gap between the k-th and (k+1)-th largest candidate score (inf if fewer than k+1)."""
    s = np.sort(_f64(scores))[::-1]
    if s.shape[0] <= k or k <= 0:
        return math.inf
    return float(s[k - 1] - s[k])


def span_extent(j: int, S: int, stride: int | None = None):
    """Token range [t0, t1) of span j.  Anchors sit every `stride` tokens (anchor of span j:
    (j+1)*stride - 1) and a span reaches S tokens back from its anchor, clipped at token 0:
    Algorithm 1's S_t = [t - b*l, t] with b*l = S.  stride = S (the default) is the disjoint grid;
    S > stride is the redundant setting of Section 2.4 / 4.4 (spans overlap their predecessors)."""
    A = S if stride is None else int(stride)
    t1 = (int(j) + 1) * A
    return max(0, t1 - S), t1


def attended_ranges(i: int, S: int, sel, stride: int | None = None):
    """The attended token set of the query at position i as disjoint ranges [t0, t1), ascending:
    the UNION of the selected spans (entries < 0 or >= c are empty slots; c = i // stride) and the
    local window [c*stride, i] -- Algorithm 1's DedupConcat: every token once, however many of the
    selected spans contain it."""
    A = S if stride is None else int(stride)
    c = i // A
    pieces = [span_extent(int(j), S, A) for j in sel if 0 <= int(j) < c]
    pieces.append((c * A, i + 1))
    pieces.sort()
    out = []
    for (t0, t1) in pieces:
        if out and t0 <= out[-1][1]:          # overlaps or touches the previous range: extend it
            out[-1] = (out[-1][0], max(out[-1][1], t1))
        else:
            out.append((t0, t1))
    return out


def attention_row(q, K, V, kv: int, i: int, S: int, sel, scale: float, return_weights=False,
                  stride: int | None = None):
    """Eq. (4) over J = union of selected spans and the local window, one joint softmax.

    K, V: anything indexable as X[kv, t0:t1] -> [t1-t0, D].  Returns (o [D], lse), fp64.
    """
    q = _f64(q)
    ks, vs = [], []
    for (t0, t1) in attended_ranges(i, S, sel, stride):
        ks.append(_f64(K[kv, t0:t1]))
        vs.append(_f64(V[kv, t0:t1]))
    Kj = np.concatenate(ks, axis=0)
    Vj = np.concatenate(vs, axis=0)
    z = scale * (Kj @ q)
    m = np.max(z)
    e = np.exp(z - m)
    l = np.sum(e)
    o = (e @ Vj) / l
    lse = m + math.log(l)
    if return_weights:
        return o, lse, e / l
    return o, lse


def span_attention(Q, K, V, idx, S: int, scale: float | None = None, q_pos0: int = 0,
                   stride: int | None = None):
    """Span-attention for every (head, query row): O [Hq, Lq, D] and LSE [Hq, Lq], fp64.

    Q: [Hq, Lq, D]; K, V: [Hkv, L, D]; idx: [Hq, Lq, k] from span_search (run with S = stride when
    the spans are longer than the anchor spacing).
    """
    Q = np.asarray(Q)
    Hq, Lq, D = Q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    O = np.zeros((Hq, Lq, D), dtype=F64)
    LSE = np.zeros((Hq, Lq), dtype=F64)
    for h in range(Hq):
        kv = h // G
        for r in range(Lq):
            o, lse = attention_row(Q[h, r], K, V, kv, q_pos0 + r, S, idx[h, r], scale, stride=stride)
            O[h, r] = o
            LSE[h, r] = lse
    return O, LSE


def merge_partials(os_, lses):
    """Log-sum-exp merge of attention partials over disjoint key sets: given each part's
    normalised output o_p and its lse_p, the joint result is sum_p w_p o_p with
    w_p = exp(lse_p - LSE), LSE = log sum_p exp(lse_p)."""
    os_ = _f64(os_)
    lses = _f64(lses)
    M = np.max(lses)
    w = np.exp(lses - M)
    tot = np.sum(w)
    return (w[:, None] * os_).sum(axis=0) / tot, M + math.log(tot)


def gate_weights(scores_sel):
    """Eq. (6): alpha = softmax over the search scores of the selected spans (fp64)."""
    s = _f64(scores_sel)
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def combined_row(q, K, V, kv: int, i: int, S: int, sel, sel_scores, scale: float, return_parts=False,
                 stride: int | None = None):
    """Algorithm 1, the per-span attention and the gate, for one query row.

    sel: selected span indices (entries < 0 or >= c are empty slots); sel_scores: the search
    score of the span in the same slot.  For every valid slot t: J_t = span t followed by the
    local window [c*S, i] (disjoint on the grid, so DedupConcat is a concatenation) and
    A_t = softmax-attention of q over J_t (eq. (4)).  O = sum_t alpha_t A_t (eq. (5)) with
    alpha from eq. (6).  No valid slot: attention over the window only.  Returns o [D] (fp64);
    with return_parts also (alpha, [A_t], valid slot numbers).  With stride < S the spans are S
    tokens long at an anchor spacing of `stride` (span_extent); a span never reaches into the
    window, and every A_t has its own softmax, so overlapping spans need no de-duplication here.
    """
    q = _f64(q)
    A_ = S if stride is None else int(stride)
    c = i // A_
    Kw, Vw = _f64(K[kv, c * A_:i + 1]), _f64(V[kv, c * A_:i + 1])
    slots = [n for n, j in enumerate(sel) if 0 <= int(j) < c]

    def attend(Kj, Vj):
        z = scale * (Kj @ q)
        e = np.exp(z - np.max(z))
        return (e @ Vj) / np.sum(e)

    if not slots:
        o = attend(Kw, Vw)
        return (o, np.zeros(0), [], []) if return_parts else o
    A = []
    for n in slots:
        t0, t1 = span_extent(int(sel[n]), S, A_)
        Kj = np.concatenate([_f64(K[kv, t0:t1]), Kw], axis=0)
        Vj = np.concatenate([_f64(V[kv, t0:t1]), Vw], axis=0)
        A.append(attend(Kj, Vj))
    alpha = gate_weights([sel_scores[n] for n in slots])
    o = np.zeros_like(A[0])
    for a, At in zip(alpha, A):
        o = o + a * At
    return (o, alpha, A, slots) if return_parts else o


def span_attention_combined(Q, K, V, idx, scores, S: int, scale: float | None = None, q_pos0: int = 0,
                            stride: int | None = None):
    """combined_row for every (head, query row): O [Hq, Lq, D], fp64.  idx, scores: [Hq, Lq, k]."""
    Q = np.asarray(Q)
    Hq, Lq, D = Q.shape
    G = Hq // K.shape[0]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    O = np.zeros((Hq, Lq, D), dtype=F64)
    for h in range(Hq):
        for r in range(Lq):
            O[h, r] = combined_row(Q[h, r], K, V, h // G, q_pos0 + r, S, idx[h, r], scores[h, r], scale,
                                   stride=stride)
    return O


# ---------------------------------------------------------------------------------------------
# The paper's own geometry (Section 3.3; Fig. 3; Algorithm 1), for one query position i:
# anchors on a quadratic stride pattern, spans of a length that grows with sqrt(i) around the
# selected anchors, a sliding window W, anchors inside W dropped.  p = 1/2 (the N = 2 case).

def anchor_positions(i: int, root: int = 2):
    """Anchor tokens of query position i for search exponent p = 1/root:
    t_s = i - (s+1)^(1/p) + 1 = i - (s+1)^root + 1, s = 0, 1, ..., as long as t_s >= 0
    (Section 3.3; for p = 1/2: "i, i-3, i-8, i-15, ...")."""
    out = []
    s = 0
    while i - (s + 1) ** root + 1 >= 0:
        out.append(i - (s + 1) ** root + 1)
        s += 1
    return out


def base_span_length(i: int, root: int = 2) -> int:
    """l(i) = ceil(i^(1-p)) for p = 1/root (Section 3.3), in exact integer arithmetic: the
    smallest integer m with m^root >= i^(root-1).  root = 2: ceil(sqrt(i)); root = 3 is the
    (1/3, 2/3) split of search and span exponents (Section 5)."""
    target = int(i) ** (root - 1)
    lo, hi = 0, max(1, int(i))          # hi^root >= i^(root-1) for every i >= 0
    while lo < hi:                      # smallest m in [0, hi] with m^root >= target
        mid = (lo + hi) // 2
        if mid ** root >= target:
            hi = mid
        else:
            lo = mid + 1
    return lo


def window_range(i: int, w: int):
    """W = [max(0, i-w+1), i] (Algorithm 1); None if w = 0."""
    return None if w <= 0 else (max(0, i - w + 1), i)


def anchor_candidates(i: int, w: int, root: int = 2):
    """T = Anchors(i) minus W (Algorithm 1): (stride index s, anchor t_s) pairs, ascending s."""
    lo = i - w + 1 if w > 0 else i + 1
    return [(s, t) for s, t in enumerate(anchor_positions(i, root)) if t < lo]


def anchor_span(t: int, i: int, b: int, f: int, root: int = 2):
    """S_t = [max(0, t - b*l(i)), min(i, t + f*l(i))] (Algorithm 1), inclusive bounds."""
    l = base_span_length(i, root)
    return max(0, t - b * l), min(i, t + f * l)


def anchor_search_row(qs, Krow, i: int, w: int, topk: int, root: int = 2):
    """Scores <Q_s(i), K_a(t)> (eq. (2), K_a = K) of the candidate anchors of position i and the
    top-k of them (eq. (3)); ties go to the lower stride index (the anchor nearer to the query).
    Krow: anything indexable as Krow[t] -> [D].  Returns (stride indices ascending, their anchor
    positions, their scores), each of length min(topk, number of candidates)."""
    cand = anchor_candidates(i, w, root)
    qs = _f64(qs)
    sc = np.array([float(_f64(Krow[t]) @ qs) for _, t in cand], dtype=F64)
    order = select_topk(sc, topk)          # ascending candidate number = ascending stride index
    return [cand[n][0] for n in order], [cand[n][1] for n in order], [float(sc[n]) for n in order]


def anchor_combined_row(q, K, V, kv: int, i: int, w: int, b: int, f: int, sel_t, sel_scores, scale: float,
                        return_parts=False, root: int = 2):
    """Algorithm 1 for one query row on the paper's geometry: for every selected anchor t,
    J_t = DedupConcat(S_t, W) (the set union, every token once), A_t = softmax attention over
    J_t (eq. (4)); O = sum_t alpha_t A_t with alpha = softmax of the selected scores (eq. (5)-(6));
    nothing selected: attention over W.  Entries of sel_t < 0 are empty slots."""
    q = _f64(q)
    W = window_range(i, w)

    def attend(tokens):
        Kj = np.stack([_f64(K[kv, t:t + 1])[0] for t in tokens])
        Vj = np.stack([_f64(V[kv, t:t + 1])[0] for t in tokens])
        z = scale * (Kj @ q)
        e = np.exp(z - np.max(z))
        return (e @ Vj) / np.sum(e)

    wtok = list(range(W[0], W[1] + 1)) if W else []
    slots = [n for n, t in enumerate(sel_t) if int(t) >= 0]
    if not slots:
        o = attend(wtok)
        return (o, np.zeros(0), []) if return_parts else o
    A = []
    for n in slots:
        a, e = anchor_span(int(sel_t[n]), i, b, f, root)
        tokens = sorted(set(range(a, e + 1)) | set(wtok))
        A.append(attend(tokens))
    alpha = gate_weights([sel_scores[n] for n in slots])
    o = np.zeros_like(A[0])
    for g, At in zip(alpha, A):
        o = o + g * At
    return (o, alpha, A) if return_parts else o
