"""Pins for the CPU oracle: every check compares oracle/ against something that is not oracle/
(brute force over the full L x L problem, library routines, closed forms, hand-derived values
under tests/golden/).  No GPU needed."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import superlinear as orc
from tests import brute

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, Hq, Hkv, L, D, Lq=None):
    rng = np.random.default_rng(seed)
    Lq = L if Lq is None else Lq
    return (rng.standard_normal((Hq, Lq, D)), rng.standard_normal((Hkv, L, D)),
            rng.standard_normal((Hkv, L, D)))


def _rows(path):
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [c.strip() for c in line.split(";")]


# ---------------------------------------------------------------- golden, hand-derived values

def test_golden_attention_closed_form():
    L, S = 6, 2
    K = np.log(np.arange(1, L + 1, dtype=np.float64)).reshape(1, L, 1)
    V = np.arange(L, dtype=np.float64).reshape(1, L, 1)
    n = 0
    for i, sel, num, den, elsE in _rows(os.path.join(GOLD, "attention_closed_form.txt")):
        i = int(i)
        sel = [] if sel == "-" else [int(x) for x in sel.split(",")]
        o, lse = orc.attention_row(np.array([1.0]), K, V, 0, i, S, sel, 1.0)
        assert o[0] == pytest.approx(int(num) / int(den), rel=1e-13, abs=1e-13)
        assert lse == pytest.approx(math.log(int(elsE)), rel=1e-13, abs=1e-13)
        n += 1
    assert n == 11


def test_golden_search_ties():
    S = 2
    Ks = np.array([[[3, 9], [5, 9], [5, -2], [1, 0], [4, 4], [5, 1]]], dtype=np.float64)
    n = 0
    for c, k, exp in _rows(os.path.join(GOLD, "search_ties.txt")):
        c, k = int(c), int(k)
        exp = [int(x) for x in exp.split(",")]
        # one query at position c*S (first token of span c): candidates are spans 0..c-1
        Qs = np.array([[[1.0, 0.0]]])
        idx = orc.span_search(Qs, Ks, S, k, q_pos0=c * S)
        assert idx.dtype == np.int32 and idx.shape == (1, 1, k)
        assert idx[0, 0].tolist() == exp
        n += 1
    assert n == 10


# ---------------------------------------------------------------- span-search pins

@pytest.mark.parametrize("seed,Hq,Hkv,L,D,S,k", [
    (0, 2, 1, 48, 8, 4, 3), (1, 4, 2, 60, 16, 5, 4), (2, 3, 3, 33, 4, 3, 12), (3, 4, 1, 64, 8, 8, 1)])
def test_search_equals_bruteforce_argsort(seed, Hq, Hkv, L, D, S, k):
    Qs, K, _ = _rand(seed, Hq, Hkv, L, D)
    Ks = orc.span_keys(K, S)
    # independent expression of the span keys: strided slice of K at the last token of each span
    assert np.array_equal(Ks, K[:, S - 1::S, :][:, :L // S])
    idx, sc = orc.span_search(Qs, Ks, S, k, return_scores=True)
    G = Hq // Hkv
    allscores = np.einsum("hqd,hjd->hqj", Qs, np.repeat(Ks, G, axis=0))   # full score matrix
    for h in range(Hq):
        for i in range(L):
            c = i // S                                   # closed form: floor(i / S) candidates
            want = brute.argsort_topk(allscores[h, i, :c], k)
            got = idx[h, i]
            assert np.array_equal(got[:len(want)], want)
            assert np.all(got[len(want):] == -1)
            assert len(want) == min(k, c)
            # every selected anchor is causal and lies below the query's own span
            assert all((j + 1) * S - 1 < c * S <= i for j in want)
            assert np.allclose(sc[h, i, :len(want)], allscores[h, i, want], rtol=1e-13)
            assert np.all(np.isneginf(sc[h, i, len(want):]))


def test_search_duplicate_keys_lower_index_wins():
    rng = np.random.default_rng(7)
    D, S, n = 8, 4, 10
    base = rng.standard_normal((3, D))
    # spans 0..9 carry one of three distinct keys -> many exact ties
    pattern = [0, 1, 0, 2, 1, 0, 2, 2, 1, 0]
    Ks = base[pattern][None]
    q = rng.standard_normal((1, 1, D))
    s = base @ q[0, 0]
    best = int(np.argmax(s))
    members = [j for j, p in enumerate(pattern) if p == best]
    for k in range(1, len(members) + 1):
        idx = orc.span_search(q, Ks, S, k, q_pos0=n * S)
        assert idx[0, 0].tolist() == members[:k]


def test_search_chunked_equals_whole():
    Qs, K, _ = _rand(11, 2, 1, 40, 8)
    Ks = orc.span_keys(K, 4)
    whole = orc.span_search(Qs, Ks, 4, 3)
    part = orc.span_search(Qs[:, 17:29], Ks, 4, 3, q_pos0=17)
    assert np.array_equal(whole[:, 17:29], part)


def test_selection_margin():
    assert orc.selection_margin([5.0, 1.0, 4.0, 3.5], 2) == pytest.approx(0.5)
    assert orc.selection_margin([5.0, 1.0], 2) == math.inf


# ---------------------------------------------------------------- span-attention pins

@pytest.mark.parametrize("seed,Hq,Hkv,L,D,S", [(0, 2, 1, 24, 8, 4), (1, 4, 2, 30, 16, 5), (2, 2, 2, 17, 4, 3)])
def test_all_spans_selected_equals_dense_causal(seed, Hq, Hkv, L, D, S):
    Q, K, V = _rand(seed, Hq, Hkv, L, D)
    n = orc.n_spans(L, S)
    idx = orc.span_search(Q, orc.span_keys(K, S), S, n)          # top-k covers every span
    scale = 0.37
    O, LSE = orc.span_attention(Q, K, V, idx, S, scale=scale)
    Od, LSEd, _ = brute.dense_masked_attention(Q, K, V, brute.causal_mask(Hq, L, L), scale)
    assert np.allclose(O, Od, rtol=1e-12, atol=1e-13)
    assert np.allclose(LSE, LSEd, rtol=1e-12, atol=1e-13)


def test_single_span_is_dense_causal_and_default_scale():
    Q, K, V = _rand(5, 2, 1, 16, 8)
    idx = np.full((2, 16, 2), -1, dtype=np.int32)
    O, LSE = orc.span_attention(Q, K, V, idx, 16)                 # S = L: one span, window = prefix
    Od, LSEd, _ = brute.dense_masked_attention(Q, K, V, brute.causal_mask(2, 16, 16), 1 / math.sqrt(8))
    assert np.allclose(O, Od, rtol=1e-12) and np.allclose(LSE, LSEd, rtol=1e-12)


def test_topk_zero_is_block_diagonal_causal_vs_torch_sdpa():
    # textbook special case reproduced by a library routine with an explicit mask
    Hq, Hkv, L, D, S = 4, 2, 24, 8, 6
    Q, K, V = _rand(9, Hq, Hkv, L, D)
    idx = np.full((Hq, L, 1), -1, dtype=np.int32)
    O, _ = orc.span_attention(Q, K, V, idx, S)
    i = torch.arange(L)[:, None]
    t = torch.arange(L)[None, :]
    mask = (t <= i) & (t // S == i // S)
    Kt = torch.from_numpy(K).repeat_interleave(Hq // Hkv, dim=0)
    Vt = torch.from_numpy(V).repeat_interleave(Hq // Hkv, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], Kt[None], Vt[None], attn_mask=mask)[0].numpy()
    assert np.allclose(O, ref, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_arbitrary_selection_equals_masked_dense(seed):
    # random (not searched) span sets, incl. empty slots and out-of-range entries that must be ignored
    Hq, Hkv, L, D, S, k = 4, 2, 40, 8, 5, 3
    Q, K, V = _rand(20 + seed, Hq, Hkv, L, D)
    rng = np.random.default_rng(seed)
    idx = np.full((Hq, L, k), -1, dtype=np.int32)
    for h in range(Hq):
        for i in range(L):
            c = i // S
            pool = list(rng.permutation(c))[:k]
            row = sorted(pool) + [-1] * (k - len(pool))
            if rng.random() < 0.3 and c < L // S:
                row[-1] = c if row[-1] == -1 else row[-1]       # own span or beyond: ignored
            idx[h, i] = row
    O, LSE = orc.span_attention(Q, K, V, idx, S, scale=0.5)
    Od, LSEd, _ = brute.dense_masked_attention(Q, K, V, brute.span_mask(idx, S, L), 0.5)
    assert np.allclose(O, Od, rtol=1e-12, atol=1e-13)
    assert np.allclose(LSE, LSEd, rtol=1e-12, atol=1e-13)


def test_weights_sum_to_one_and_key_count_closed_form():
    Hq, Hkv, L, D, S, k = 2, 1, 50, 8, 5, 3
    Q, K, V = _rand(3, Hq, Hkv, L, D)
    idx = orc.span_search(Q, orc.span_keys(K, S), S, k)
    for h in range(Hq):
        for i in range(L):
            o, lse, w = orc.attention_row(Q[h, i], K, V, 0, i, S, idx[h, i], 0.3, return_weights=True)
            assert w.sum() == pytest.approx(1.0, abs=1e-14)
            assert np.all(w > 0)
            # attended keys = min(k, c) * S + (i mod S) + 1
            assert w.shape[0] == min(k, i // S) * S + (i % S) + 1


def test_slot_permutation_invariance():
    Hq, Hkv, L, D, S, k = 2, 2, 48, 8, 4, 4
    Q, K, V = _rand(4, Hq, Hkv, L, D)
    idx = orc.span_search(Q, orc.span_keys(K, S), S, k)
    O, LSE = orc.span_attention(Q, K, V, idx, S)
    rng = np.random.default_rng(0)
    perm = idx.copy()
    for h in range(Hq):
        for i in range(L):
            perm[h, i] = idx[h, i][rng.permutation(k)]
    O2, LSE2 = orc.span_attention(Q, K, V, perm, S)
    assert np.allclose(O, O2, rtol=1e-13, atol=1e-14) and np.allclose(LSE, LSE2, rtol=1e-13)


def test_identical_keys_give_mean_of_values():
    # closed form: if every key is the same vector the weights are uniform over J
    Hq, Hkv, L, D, S, k = 1, 1, 32, 4, 4, 2
    rng = np.random.default_rng(1)
    kvec = rng.standard_normal(D)
    K = np.broadcast_to(kvec, (1, L, D)).copy()
    V = rng.standard_normal((1, L, D))
    Q = rng.standard_normal((1, L, D))
    idx = orc.span_search(Q, orc.span_keys(K, S), S, k)      # all ties -> lowest spans
    O, LSE = orc.span_attention(Q, K, V, idx, S, scale=1.0)
    for i in range(L):
        c = i // S
        sel = list(range(min(k, c)))
        assert idx[0, i, :len(sel)].tolist() == sel
        toks = [t for j in sel for t in range(j * S, (j + 1) * S)] + list(range(c * S, i + 1))
        assert np.allclose(O[0, i], V[0, toks].mean(axis=0), rtol=1e-12)
        assert LSE[0, i] == pytest.approx(float(Q[0, i] @ kvec) + math.log(len(toks)), rel=1e-12)


def test_gqa_head_mapping():
    # head h must read kv head h // G (not h % Hkv): make kv heads wildly different
    Hq, Hkv, L, D, S = 4, 2, 12, 4, 4
    Q, K, V = _rand(8, Hq, Hkv, L, D)
    V[1] += 100.0
    idx = np.full((Hq, L, 1), -1, dtype=np.int32)
    O, _ = orc.span_attention(Q, K, V, idx, S)
    assert np.all(np.abs(O[0:2]) < 50) and np.all(O[2:4] > 50)


def test_attention_chunked_equals_whole():
    Hq, Hkv, L, D, S, k = 2, 1, 36, 8, 4, 2
    Q, K, V = _rand(12, Hq, Hkv, L, D)
    idx = orc.span_search(Q, orc.span_keys(K, S), S, k)
    O, LSE = orc.span_attention(Q, K, V, idx, S)
    O2, LSE2 = orc.span_attention(Q[:, 13:30], K, V, idx[:, 13:30], S, q_pos0=13)
    assert np.array_equal(O[:, 13:30], O2) and np.array_equal(LSE[:, 13:30], LSE2)


def test_merge_partials_identity():
    # merging per-span partials equals the one-shot softmax over the union (textbook identity)
    Hq, Hkv, L, D, S = 1, 1, 40, 8, 8
    Q, K, V = _rand(13, Hq, Hkv, L, D)
    i, sel, scale = 37, [0, 2, 3], 0.4
    o_all, lse_all = orc.attention_row(Q[0, i], K, V, 0, i, S, sel, scale)
    parts_o, parts_l = [], []
    for (t0, t1) in orc.attended_ranges(i, S, sel):
        Od, Ld, _ = brute.dense_masked_attention(
            Q[:, i:i + 1], K[:, t0:t1], V[:, t0:t1], np.ones((1, 1, t1 - t0), bool), scale)
        parts_o.append(Od[0, 0])
        parts_l.append(Ld[0, 0])
    o, lse = orc.merge_partials(np.stack(parts_o), np.array(parts_l))
    assert np.allclose(o, o_all, rtol=1e-12) and lse == pytest.approx(lse_all, rel=1e-13)


def test_random_context_access_cover():
    # structural non-exclusion (Section 2.3) on the grid: candidate spans plus the local window
    # cover every key position j <= i
    for S in (1, 3, 8):
        for i in range(0, 70):
            c = i // S
            cover = set()
            for (t0, t1) in orc.attended_ranges(i, S, list(range(c))):
                cover |= set(range(t0, t1))
            assert cover == set(range(i + 1))


# ---------------------------------------------------------------- combination (Section 3.4, eq. (5)-(6))

def _searched(seed, Hq, Hkv, L, D, S, k):
    Q, K, V = _rand(seed, Hq, Hkv, L, D)
    idx, sc = orc.span_search(Q, orc.span_keys(K, S), S, k, return_scores=True)
    return Q, K, V, idx, sc


@pytest.mark.parametrize("seed,Hq,Hkv,L,D,S,k", [(0, 4, 2, 40, 8, 5, 3), (1, 2, 1, 33, 4, 4, 8), (2, 3, 3, 24, 8, 6, 1)])
def test_combination_equals_dense_per_slot_bruteforce(seed, Hq, Hkv, L, D, S, k):
    # one full masked softmax per slot + library softmax over the slot scores
    Q, K, V, idx, sc = _searched(30 + seed, Hq, Hkv, L, D, S, k)
    O = orc.span_attention_combined(Q, K, V, idx, sc, S, scale=0.4)
    Ob, alpha = brute.gated_combination(Q, K, V, idx, sc, S, 0.4)
    assert np.allclose(O, Ob, rtol=1e-12, atol=1e-13)
    # gate weights of every row with a selection sum to one
    has = (idx >= 0).any(axis=-1)
    assert np.allclose(alpha.sum(-1)[has], 1.0, atol=1e-14)


def test_combination_with_one_span_is_the_joint_softmax():
    # k = 1: alpha = 1 and J_t = span | window is the whole attended set, so the gated output is
    # eq. (4) over that set -- the same masked dense attention that pins attention_row
    Hq, Hkv, L, D, S = 2, 1, 36, 8, 6
    Q, K, V, idx, sc = _searched(40, Hq, Hkv, L, D, S, 1)
    O = orc.span_attention_combined(Q, K, V, idx, sc, S, scale=0.7)
    Od, _, _ = brute.dense_masked_attention(Q, K, V, brute.span_mask(idx, S, L), 0.7)
    assert np.allclose(O, Od, rtol=1e-12, atol=1e-13)


def test_combination_empty_selection_is_window_attention():
    # rows of the first span have no candidate: Algorithm 1's window-only branch = block-diagonal causal
    Hq, Hkv, L, D, S = 2, 2, 12, 4, 6
    Q, K, V = _rand(41, Hq, Hkv, L, D)
    idx = np.full((Hq, L, 2), -1, dtype=np.int32)
    sc = np.full((Hq, L, 2), -np.inf)
    O = orc.span_attention_combined(Q, K, V, idx, sc, S, scale=0.5)
    Od, _, _ = brute.dense_masked_attention(Q, K, V, brute.span_mask(idx, S, L), 0.5)
    assert np.allclose(O, Od, rtol=1e-12, atol=1e-13)


def test_gate_weights_closed_forms():
    # equal scores -> uniform; two scores -> logistic of their difference; shift invariance
    assert np.allclose(orc.gate_weights([2.5, 2.5, 2.5, 2.5]), 0.25)
    a = orc.gate_weights([1.0, 3.0])
    assert a[1] == pytest.approx(1.0 / (1.0 + math.exp(-2.0)), abs=1e-15)
    assert a.sum() == pytest.approx(1.0, abs=1e-15)
    assert np.allclose(orc.gate_weights([1.0, 3.0, -2.0]), orc.gate_weights([101.0, 103.0, 98.0]), atol=1e-15)
    # the scores are used as they are (no 1/sqrt(D), eq. (6)): a gap of 50 saturates the gate
    assert orc.gate_weights([50.0, 0.0])[0] == pytest.approx(1.0, abs=1e-20)


def test_combination_equal_scores_is_mean_of_span_outputs_and_slot_order_free():
    Hq, Hkv, L, D, S, k = 1, 1, 40, 8, 5, 3
    Q, K, V = _rand(42, Hq, Hkv, L, D)
    i, sel = 37, [1, 4, 6]
    o, alpha, A, slots = orc.combined_row(Q[0, i], K, V, 0, i, S, sel, [0.3, 0.3, 0.3], 0.5, return_parts=True)
    assert np.allclose(alpha, 1 / 3) and slots == [0, 1, 2]
    assert np.allclose(o, np.mean(A, axis=0), rtol=1e-13)
    # each A_t is the one-span attention (masked dense over span | window)
    for t, At in zip(sel, A):
        ref, _, _ = brute.dense_masked_attention(Q[:, i:i + 1], K, V,
                                                brute.span_mask(np.array([[[t]]]), S, L, q_pos0=i), 0.5)
        assert np.allclose(At, ref[0, 0], rtol=1e-12, atol=1e-13)
    # permuting the slots together with their scores changes nothing; empty slots are skipped
    o1 = orc.combined_row(Q[0, i], K, V, 0, i, S, [6, -1, 1, 4], [0.9, 123.0, -0.2, 0.1], 0.5)
    o2 = orc.combined_row(Q[0, i], K, V, 0, i, S, [1, 4, 6, 7], [-0.2, 0.1, 0.9, 55.0], 0.5)  # 7 = c, the query's own span: empty
    o3 = orc.combined_row(Q[0, i], K, V, 0, i, S, [9, 1, 4, 6], [7.0, -0.2, 0.1, 0.9], 0.5)   # beyond the cache: empty
    assert np.allclose(o1, o3, rtol=1e-13, atol=1e-14)
    assert np.allclose(o1, o2, rtol=1e-13, atol=1e-14)


def test_combination_identical_spans_collapse():
    # if every selected span holds the same keys and values, all A_t coincide and O = A_t whatever the gate
    Hq, Hkv, L, D, S = 1, 1, 30, 4, 5
    Q, K, V = _rand(43, Hq, Hkv, L, D)
    for j in (1, 2):
        K[0, j * S:(j + 1) * S] = K[0, 0:S]
        V[0, j * S:(j + 1) * S] = V[0, 0:S]
    i = 28
    o = orc.combined_row(Q[0, i], K, V, 0, i, S, [0, 1, 2], [5.0, -1.0, 0.2], 0.6)
    one = orc.combined_row(Q[0, i], K, V, 0, i, S, [2], [0.0], 0.6)
    assert np.allclose(o, one, rtol=1e-13, atol=1e-14)


# ---------------------------------------------------------------- the paper's own geometry (Section 3.3, Fig. 3)

def _gold_geometry():
    g = {}
    for kind, vals in _rows(os.path.join(GOLD, "anchor_geometry.txt")):
        g[kind] = [int(v) for v in vals.split(",")]
    return g


def test_golden_fig3_anchors_span_length_and_cover():
    g = _gold_geometry()
    i, b, f = g["fig3_i"][0], g["fig3_b"][0], g["fig3_f"][0]
    assert orc.anchor_positions(i) == g["fig3_anchors"]
    assert (b + f) * orc.base_span_length(i) == g["fig3_span_length"][0]
    # every position 0..i lies in at least one candidate span (no window in the figure)
    covered = set()
    for t in orc.anchor_positions(i):
        a, e = orc.anchor_span(t, i, b, f)
        assert e == t and t - a == min(t, g["fig3_span_length"][0])      # f = 0: the span ends at its anchor
        covered |= set(range(a, e + 1))
    assert covered == set(range(i + 1))


def test_golden_anchor_offsets_and_gaps():
    g = _gold_geometry()
    for i in (15, 100, 4097):
        a = orc.anchor_positions(i)
        assert [i - t for t in a[:4]] == g["text_offsets"]
        assert [a[n] - a[n + 1] for n in range(3)] == g["text_gaps"]


@pytest.mark.parametrize("i", [0, 1, 2, 3, 8, 24, 99, 1000, 65535, 1048575])
def test_anchor_count_and_base_length_closed_forms(i):
    a = orc.anchor_positions(i)
    assert len(a) == math.isqrt(i + 1)                 # (s+1)^2 <= i + 1
    assert a[0] == i and all(x > y for x, y in zip(a, a[1:])) and a[-1] >= 0
    l = orc.base_span_length(i)
    assert (l - 1) ** 2 < max(i, 1) <= l * l or i == 0 and l == 0
    assert l == math.ceil(math.sqrt(i)) or i > 2 ** 40   # float sqrt is exact enough at these sizes


@pytest.mark.parametrize("i,w,b", [(30, 0, 2), (500, 48, 2), (4095, 99, 2), (100000, 1088, 4)])
def test_random_context_access_on_paper_geometry(i, w, b):
    # Section 3.3: with b >= 1/p = 2 every key j <= i is reachable: it lies in W or in the span of a
    # candidate.  The window is "chosen based on the stride index" so that the search starts right
    # after it: w = m^2 - 1 (the paper's 1088 = 33^2 - 1), the first candidate anchor is i - w.
    covered = set()
    W = orc.window_range(i, w)
    if W:
        covered |= set(range(W[0], W[1] + 1))
    cand = orc.anchor_candidates(i, w)
    assert W is None or cand[0][1] == W[0] - 1
    for _, t in cand:
        assert W is None or t < W[0]
        a, e = orc.anchor_span(t, i, b, 0)
        covered |= set(range(a, e + 1))
    assert covered == set(range(i + 1))


@pytest.mark.parametrize("i", [0, 1, 6, 7, 8, 26, 27, 999, 1000, 262143, 10 ** 6])
def test_anchor_closed_forms_for_one_third_two_thirds(i):
    # the general-p formulas of Section 3.3 at p = 1/3: anchors i - (s+1)^3 + 1 (offsets 0, 7, 26,
    # 63, ...; gaps 3s^2 + 9s + 7), floor((i+1)^(1/3)) of them; l(i) = ceil(i^(2/3)), the exponent
    # split (1/3, 2/3) of Section 5
    a = orc.anchor_positions(i, 3)
    n = len(a)
    assert n ** 3 <= i + 1 < (n + 1) ** 3
    assert [i - t for t in a] == [(s + 1) ** 3 - 1 for s in range(n)]
    assert [a[s] - a[s + 1] for s in range(n - 1)] == [3 * s * s + 9 * s + 7 for s in range(n - 1)]
    l = orc.base_span_length(i, 3)
    assert l ** 3 >= i * i and (l == 0 or (l - 1) ** 3 < i * i)
    if 0 < i < 10 ** 5:
        assert abs(l - i ** (2.0 / 3.0)) < 1.0 + 1e-6


@pytest.mark.parametrize("i,w", [(200, 0), (5000, 26), (100000, 342)])
def test_random_context_access_for_one_third_two_thirds(i, w):
    # b >= 1/p = 3 reaches every key (Section 3.3): gaps between adjacent anchors are at most
    # 3 (s+1)^2 + 3 (s+1) + 1 <= 3 i^(2/3) for (s+2)^3 <= i + 1.  Windows w = m^3 - 1 put the first
    # candidate right before W.
    covered = set()
    W = orc.window_range(i, w)
    if W:
        covered |= set(range(W[0], W[1] + 1))
    cand = orc.anchor_candidates(i, w, 3)
    assert W is None or cand[0][1] == W[0] - 1
    for _, t in cand:
        a, e = orc.anchor_span(t, i, 3, 0, 3)
        covered |= set(range(a, e + 1))
    assert covered == set(range(i + 1))
    # ... and b = 2 is not enough there
    short = set(range(W[0], W[1] + 1)) if W else set()
    for _, t in cand:
        a, e = orc.anchor_span(t, i, 2, 0, 3)
        short |= set(range(a, e + 1))
    assert short != set(range(i + 1))


def test_anchor_search_equals_bruteforce_argsort():
    rng = np.random.default_rng(50)
    i, w, k, D = 777, 50, 4, 8
    K = rng.standard_normal((i + 1, D))
    q = rng.standard_normal(D)
    s_sel, t_sel, sc_sel = orc.anchor_search_row(q, K, i, w, k)
    cand_t = [t for t in (i - (s + 1) ** 2 + 1 for s in range(100)) if 0 <= t < i - w + 1]
    scores = K[cand_t] @ q
    want = brute.argsort_topk(scores, k)
    assert t_sel == [cand_t[n] for n in want]
    assert np.allclose(sc_sel, scores[want], rtol=1e-13)
    assert s_sel == sorted(s_sel) and t_sel == sorted(t_sel, reverse=True)
    # a duplicated key: the nearer anchor (lower stride index) wins the tie
    K2 = K.copy()
    K2[cand_t[5]] = K2[cand_t[2]] = 10.0 * q
    s2, t2, _ = orc.anchor_search_row(q, K2, i, w, 1)
    assert t2 == [cand_t[2]]


def test_anchor_combined_equals_dense_masked_bruteforce():
    # per selected anchor one dense masked softmax over (S_t | W), gate by a library softmax
    rng = np.random.default_rng(51)
    L, D, w, b, f, k = 400, 8, 30, 4, 2, 3
    i = L - 1
    Q = rng.standard_normal((1, 1, D))
    K = rng.standard_normal((1, L, D))
    V = rng.standard_normal((1, L, D))
    _, t_sel, sc_sel = orc.anchor_search_row(Q[0, 0], K[0], i, w, k)
    o, alpha, A = orc.anchor_combined_row(Q[0, 0], K, V, 0, i, w, b, f, t_sel, sc_sel, 0.5, return_parts=True)
    from scipy.special import softmax as sp_softmax
    l = math.ceil(math.sqrt(i))
    want = np.zeros(D)
    a_ref = sp_softmax(np.array(sc_sel))
    for g, t in zip(a_ref, t_sel):
        mask = np.zeros((1, 1, L), dtype=bool)
        mask[0, 0, max(0, t - b * l):min(i, t + f * l) + 1] = True      # spans of close anchors overlap: fine, each has its own softmax
        mask[0, 0, i - w + 1:i + 1] = True
        At, _, _ = brute.dense_masked_attention(Q, K, V, mask, 0.5)
        want += g * At[0, 0]
    assert np.allclose(alpha, a_ref, atol=1e-15)
    assert np.allclose(o, want, rtol=1e-12, atol=1e-13)
    # nothing selected -> window attention
    o0 = orc.anchor_combined_row(Q[0, 0], K, V, 0, i, w, b, f, [-1, -1], [0.0, 0.0], 0.5)
    mask = np.zeros((1, 1, L), dtype=bool)
    mask[0, 0, i - w + 1:i + 1] = True
    Aw, _, _ = brute.dense_masked_attention(Q, K, V, mask, 0.5)
    assert np.allclose(o0, Aw[0, 0], rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- redundant grid: spans longer than the anchor
# spacing (Section 2.4: p_sh + p_sp > 1; Section 4.4's redundancy factors), de-duplicated union

def test_redundant_spans_extent_and_union_closed_forms():
    # anchors every A = 4 tokens, spans S = 12 tokens long: span j = [max(0, 4(j+1) - 12), 4(j+1))
    A, S = 4, 12
    assert orc.span_extent(0, S, A) == (0, 4) and orc.span_extent(1, S, A) == (0, 8)
    assert orc.span_extent(2, S, A) == (0, 12) and orc.span_extent(5, S, A) == (12, 24)
    assert orc.span_extent(3, S) == (36, 48)                        # stride = S: the disjoint grid
    i = 41                                                          # cell c = 10, window [40, 41]
    # spans 4 = [8, 20) and 5 = [12, 24) overlap in [12, 20): union [8, 24); span 8 = [24, 36) touches it
    assert orc.attended_ranges(i, S, [4, 5, -1], A) == [(8, 24), (40, 42)]
    assert orc.attended_ranges(i, S, [5, 4, 8], A) == [(8, 36), (40, 42)]
    assert orc.attended_ranges(i, S, [9, 10, 11], A) == [(28, 42)]   # span 9 = [28, 40) meets the window; 10, 11 are not candidates
    # attended keys of consecutive selections j .. j+m-1 (start >= 0): S + (m-1)*A, plus the window
    Q, K, V = _rand(7, 1, 1, 64, 4)
    for m in (1, 2, 3, 5):
        sel = list(range(3, 3 + m))
        o, lse, w = orc.attention_row(Q[0, 63], K, V, 0, 63, S, sel, 0.5, return_weights=True, stride=A)
        assert w.shape[0] == S + (m - 1) * A + 4 and w.sum() == pytest.approx(1.0, abs=1e-14)


@pytest.mark.parametrize("seed,A,S", [(0, 5, 10), (1, 4, 12), (2, 3, 7), (3, 6, 6)])
def test_redundant_spans_equal_masked_dense(seed, A, S):
    # random selections on the anchor grid, incl. neighbours (overlapping spans), empty and garbage slots
    Hq, Hkv, L, D, k = 4, 2, 61, 8, 4
    Q, K, V = _rand(50 + seed, Hq, Hkv, L, D)
    rng = np.random.default_rng(seed)
    idx = np.full((Hq, L, k), -1, dtype=np.int32)
    for h in range(Hq):
        for i in range(L):
            c = i // A
            pool = list(rng.permutation(c))[:k]
            row = pool + [-1] * (k - len(pool))
            if rng.random() < 0.3:
                row[-1] = c + int(rng.integers(0, 2))               # own cell or beyond: ignored
            idx[h, i] = row
    O, LSE = orc.span_attention(Q, K, V, idx, S, scale=0.5, stride=A)
    Od, LSEd, _ = brute.dense_masked_attention(Q, K, V, brute.span_mask(idx, S, L, stride=A), 0.5)
    assert np.allclose(O, Od, rtol=1e-12, atol=1e-13)
    assert np.allclose(LSE, LSEd, rtol=1e-12, atol=1e-13)


def test_redundant_spans_all_selected_is_dense_causal():
    # every anchor selected: the overlapping spans and the window cover [0, i] exactly once each
    Hq, Hkv, L, D, A, S = 2, 1, 50, 8, 4, 12
    Q, K, V = _rand(8, Hq, Hkv, L, D)
    n = -(-L // A)
    idx = orc.span_search(Q, orc.span_keys(K, A), A, n)             # the search runs on the anchor grid
    O, LSE = orc.span_attention(Q, K, V, idx, S, stride=A)
    Od, LSEd, _ = brute.dense_masked_attention(Q, K, V, brute.causal_mask(Hq, L, L), 1.0 / math.sqrt(D))
    assert np.allclose(O, Od, rtol=1e-12, atol=1e-13) and np.allclose(LSE, LSEd, rtol=1e-12, atol=1e-13)


def test_redundant_spans_combination_equals_dense_per_slot_bruteforce():
    Hq, Hkv, L, D, A, S, k = 4, 2, 47, 8, 4, 10, 3
    Q, K, V = _rand(9, Hq, Hkv, L, D)
    idx, sc = orc.span_search(Q, orc.span_keys(K, A), A, k, return_scores=True)
    O = orc.span_attention_combined(Q, K, V, idx, sc, S, scale=0.4, stride=A)
    Ob, _ = brute.gated_combination(Q, K, V, idx, sc, S, 0.4, stride=A)
    assert np.allclose(O, Ob, rtol=1e-12, atol=1e-13)
