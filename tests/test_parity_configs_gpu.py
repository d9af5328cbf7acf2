"""GPU parity at the benchmark configurations' full sizes, in the launch configuration the
benchmark times.  Prefill outputs are compared with the oracle on a seeded sample of rows
(first rows, span boundaries, last rows, rows after planted needles, 2000 random positions) and
their span selection on ALL rows with a library fp64 matmul and stable sort; decode steps are
compared on every head.  The needle configuration is additionally checked on all rows through a
property that needs no oracle (selected spans must be needles when enough are eligible)."""
import numpy as np
import pytest
import torch

from oracle import superlinear as orc
from paper_2601_18401_amd import binding as B
from paper_2601_18401_amd import workloads as W
import math

from tests import brute
from tests.test_parity_gpu import (DEV, TOL, DevKV, DevRows, GatheredRows, check_anchor_row, check_attention, check_combined,
                                   check_idx, f64)

pytestmark = pytest.mark.gpu


def sample_rows(cfg, data, n_random=2000, seed=0):
    """(head, row) pairs: first rows, span boundaries, last rows, rows after planted needles on four
    heads, plus n_random seeded positions on two heads each (all heads get their share)."""
    rng = np.random.default_rng(seed)
    S, L = cfg.S, cfg.L
    pos = {0, 1, S - 1, S, S + 1, 2 * S - 1, 2 * S, L - 1, L - S, L - S - 1, (cfg.topk + 1) * S, cfg.topk * S - 1}
    if "needle_spans" in data:
        for j in data["needle_spans"].tolist():
            pos |= {min(L - 1, (j + 1) * S), min(L - 1, (j + 1) * S + 17)}
    pos = sorted(p for p in pos if 0 <= p < L)
    heads = sorted({0, cfg.Hq - 1, int(rng.integers(0, cfg.Hq)), int(rng.integers(0, cfg.Hq))})
    rows = {(h, r) for h in heads for r in pos}
    for r in rng.choice(L, size=n_random, replace=False).tolist():
        h0 = int(rng.integers(0, cfg.Hq))
        rows |= {(h0, r), ((h0 + 1 + int(rng.integers(0, cfg.Hq - 1))) % cfg.Hq, r)}
    return sorted(rows)


def run_prefill_config(name):
    cfg = W.CONFIGS[name]
    data = W.generate(cfg, device=DEV)
    Q, K, V = data["Q"], data["K"], data["V"]
    Ks = B.sl_span_keys(K, cfg.S)
    idx = B.sl_span_search_prefill(data["Qs"], K, Ks, cfg.S, cfg.topk)
    torch.cuda.synchronize()
    # every row: the selection against a library fp64 matmul + stable sort, with the validity of
    # rows that differ inside the tie margin (picked / dropped spans within the margin of the k-th)
    nrows, differ = brute.check_selection_all_rows(idx, data["Qs"], Ks, cfg.S, cfg.topk, margin=1e-3)
    print(f"[{name}] all {nrows} rows checked, {differ} differ from the stable-sort selection inside the margin")
    assert differ <= nrows // 1000
    # sampled rows against the oracle (host copies: the oracle slices K and V span by span)
    rows = sample_rows(cfg, data)
    assert len({r for _, r in rows}) >= 2000
    Qs_h, Ks_h, idx_h = data["Qs"].cpu(), Ks.cpu(), idx.cpu()
    amb = check_idx(idx_h, Qs_h, Ks_h, cfg.S, cfg.topk, 0, rows)
    print(f"[{name}] {len(rows)} sampled rows against the oracle, {amb} inside the tie margin")
    assert amb <= 3
    # attention on the oracle's indices for the sampled rows (other rows keep the GPU indices)
    Ksn = f64(Ks_h)
    idx_o = idx_h.clone()
    G = cfg.Hq // cfg.Hkv
    for (h, r) in rows:
        s = orc.search_scores_row(f64(Qs_h[h, r]), Ksn[h // G], r // cfg.S)
        sel = orc.select_topk(s, cfg.topk)
        idx_o[h, r] = torch.tensor(sel + [-1] * (cfg.topk - len(sel)), dtype=torch.int32)
    idx_o = idx_o.to(DEV)
    O, LSE = B.sl_span_attention_prefill(Q, K, V, idx_o, cfg.S)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all() and torch.isfinite(LSE).all()
    worst = check_attention(O.cpu(), LSE.cpu(), Q.cpu(), K.cpu(), V.cpu(), idx_o.cpu(), cfg.S, 0, 0.0, rows)
    print(f"[{name}] attention on {len(rows)} rows: max abs error {worst:.3e}")
    return cfg, data, idx


def test_config2_prefill_65k():
    run_prefill_config("C2")


def test_config4_prefill_262k_needles():
    cfg, data, idx = run_prefill_config("C4")
    # Property on all 8.39 M rows: with E(i) = number of needle spans below the query's span,
    # E >= k  ->  every selected span is a needle;  E < k -> all E needles are selected.
    needles = data["needle_spans"].to(DEV)
    is_needle = torch.zeros(cfg.n_spans + 1, dtype=torch.bool, device=DEV)
    is_needle[needles] = True
    c = (torch.arange(cfg.L, device=DEV) // cfg.S)                      # [L]
    E = (needles[None, :] < c[:, None]).sum(dim=1)                      # [L]
    for h in range(cfg.Hq):
        sel = idx[h].long()                                             # [L, k]
        valid = sel >= 0
        hit = is_needle[sel.clamp(min=0)] & valid
        nh = hit.sum(dim=1)
        assert torch.equal(nh, torch.minimum(E, torch.tensor(cfg.topk, device=DEV)))
        assert torch.equal(valid.sum(dim=1), torch.minimum(c, torch.tensor(cfg.topk, device=DEV)))


def test_config2_prefill_combined_65k():
    # the combination form (Section 3.4) at config 2's size, on the library's own indices and scores
    cfg = W.CONFIGS["C2"]
    data = W.generate(cfg, device=DEV)
    Q, K, V = data["Q"], data["K"], data["V"]
    Ks = B.sl_span_keys(K, cfg.S)
    idx, sc = B.sl_span_search_prefill(data["Qs"], K, Ks, cfg.S, cfg.topk, want_scores=True)
    sc = torch.where(torch.isfinite(sc), sc, torch.zeros_like(sc))
    O = B.sl_span_attention_combined_prefill(Q, K, V, idx, sc, cfg.S)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()
    check_combined(O, Q, K, V, idx, sc, cfg.S, 0, 0.0, sample_rows(cfg, data, n_random=300))


def test_config2_prefill_redundant_spans_65k():
    # config 2 with anchors every 128 tokens and spans 256 tokens long (what bench.py's
    # redundant_spans line runs): all-row selection check on the anchor grid, sampled rows against
    # the oracle's de-duplicated union
    cfg = W.CONFIGS["C2"]
    A = cfg.S // 2
    data = W.generate(cfg, device=DEV)
    Q, K, V = data["Q"], data["K"], data["V"]
    Ks = B.sl_span_keys(K, A)
    idx = B.sl_span_search_prefill(data["Qs"], K, Ks, A, cfg.topk)
    O, LSE = B.sl_span_attention_prefill(Q, K, V, idx, cfg.S, span_stride=A)
    torch.cuda.synchronize()
    nrows, differ = brute.check_selection_all_rows(idx, data["Qs"], Ks, A, cfg.topk, margin=1e-3)
    print(f"[C2, anchors every {A}] all {nrows} rows checked, {differ} differ inside the margin")
    assert differ <= nrows // 1000
    rows = sample_rows(cfg, data, n_random=500)
    worst = check_attention(O.cpu(), LSE.cpu(), Q.cpu(), K.cpu(), V.cpu(), idx.cpu(), cfg.S, 0, 0.0, rows, stride=A)
    print(f"[C2, anchors every {A}] attention on {len(rows)} rows: max abs error {worst:.3e}")


@pytest.fixture(scope="module", params=["C3", "C5"])
def decode_cache(request):
    """A decode configuration's full cache with two queries, generated once for the tests that use it
    (pytest runs them back to back per configuration) and freed afterwards."""
    name = request.param
    data = W.generate(W.CONFIGS[name], device=DEV, n_queries=2)
    yield name, data
    data.clear()
    torch.cuda.empty_cache()


def test_decode_configs_full_cache(decode_cache):
    name, data = decode_cache
    cfg = W.CONFIGS[name]
    K, V = data["K"], data["V"]
    Ks = B.sl_span_keys(K, cfg.S)
    for qi in range(2):
        Q = data["Q"][qi]
        idx = B.sl_span_search_decode(Q, K, Ks, cfg.S, cfg.topk)
        idx_k = B.sl_span_search_decode(Q, K, None, cfg.S, cfg.topk)
        torch.cuda.synchronize()
        assert torch.equal(idx, idx_k)
        check_idx(idx, Q, Ks, cfg.S, cfg.topk, cfg.L - 1)
        idx_o = torch.from_numpy(orc.span_search(f64(Q), f64(Ks), cfg.S, cfg.topk, q_pos0=cfg.L - 1)).to(DEV)
        O, LSE = B.sl_span_attention_decode(Q, K, V, idx_o, cfg.S)
        torch.cuda.synchronize()
        check_attention(O, LSE, Q, K, V, idx_o, cfg.S, cfg.L - 1, 0.0)
        if qi == 0 and name == "C3":   # the combination form on the same step (a few heads: the oracle is slow)
            idx_g, sc_g = B.sl_span_search_decode(Q, K, Ks, cfg.S, cfg.topk, want_scores=True)
            Oc = B.sl_span_attention_combined_decode(Q, K, V, idx_g, sc_g, cfg.S)
            torch.cuda.synchronize()
            check_combined(Oc, Q, K, V, idx_g, sc_g, cfg.S, cfg.L - 1, 0.0, [(0, 0), (13, 0), (31, 0)])


def test_batched_decode_at_the_benchmark_configuration():
    """8 sequences with caches of about 1M tokens each, as bench.py's batched_decode line runs them:
    every sequence against the oracle (search on every head, attention on the batch's indices)."""
    cfg = W.CONFIGS["C3"]
    data = W.generate(cfg, device=DEV, n_queries=8)
    K, V = data["K"], data["V"]
    NB = 8
    lens = [cfg.L - b * (cfg.S + 37) for b in range(NB)]
    Kc = [K.clone()[:, :lens[b]] for b in range(NB)]
    Vc = [V.clone()[:, :lens[b]] for b in range(NB)]
    Ksc = [B.sl_span_keys(Kc[b], cfg.S) for b in range(NB)]
    Qs = [data["Q"][b] for b in range(NB)]
    batch = B.DecodeBatch(Qs, Qs, Kc, Vc, Ksc, cfg.S, cfg.topk)
    idx = B.sl_span_search_decode_batched(batch)
    O, LSE = B.sl_span_attention_decode_batched(batch)
    torch.cuda.synchronize()
    for b in range(NB):
        amb = check_idx(idx[b], Qs[b], Ksc[b], cfg.S, cfg.topk, lens[b] - 1)
        assert amb <= 2                                    # rows whose k / k+1 margin is below 1e-3
        check_attention(O[b], LSE[b], Qs[b], Kc[b], Vc[b], idx[b], cfg.S, lens[b] - 1, 0.0)
    del data, K, V, Kc, Vc
    torch.cuda.empty_cache()


def test_paper_geometry_decode_at_full_cache(decode_cache):
    # the configuration's cache with the paper's kernel configuration (window 1088, top-2, b = 4, f = 2);
    # 1M: 128-token chunks, shared rows computed from registers; 10M: 256-token chunks, shared rows re-read
    name, data = decode_cache
    cfg = W.CONFIGS[name]
    K, V, Q = data["K"], data["V"], data["Q"][0]
    w, k, b, f = 1088, 2, 4, 2
    i = cfg.L - 1
    G = cfg.Hq // cfg.Hkv
    anchors, sc = B.sl_anchor_search_decode(Q, K, k, w, want_scores=True)
    O = B.sl_anchor_attention_decode(Q, K, V, anchors, sc, w, b, f)
    torch.cuda.synchronize()
    an, scn, Qn, On = anchors.cpu().numpy(), sc.cpu().numpy().astype(np.float64), f64(Q), f64(O)
    Kd, Vd = DevKV(K), DevKV(V)
    cand = orc.anchor_candidates(i, w)
    krows = [GatheredRows(K[kvh], [t for _, t in cand]) for kvh in range(cfg.Hkv)]   # the candidates' key rows
    # every head at 1M; at 10M (19K-token spans through the fp64 oracle) every head of the first and the last group
    heads = range(cfg.Hq) if name == "C3" else list(range(G)) + list(range(cfg.Hq - G, cfg.Hq))
    for h in heads:
        _, t_o, _ = orc.anchor_search_row(Qn[h, 0], krows[h // G], i, w, k)
        if an[h, 0].tolist() != t_o + [-1] * (k - len(t_o)):
            allsc = [float(krows[h // G][t] @ Qn[h, 0]) for _, t in cand]
            check_anchor_row(an[h, 0].tolist(), t_o + [-1] * (k - len(t_o)), cand, allsc, k, h)
        o = orc.anchor_combined_row(Qn[h, 0], Kd, Vd, h // G, i, w, b, f, an[h, 0], scn[h, 0], 1.0 / math.sqrt(cfg.D))
        assert float(np.max(np.abs(On[h, 0] - o))) <= TOL[torch.bfloat16]
    # the heads of every group on neighbouring anchors: their spans overlap almost entirely without
    # being equal, so most chunks are read by one workgroup for several (head, slot) entries
    rng = np.random.default_rng(7)
    an2 = np.empty((cfg.Hq, 1, k), np.int32)
    sc2 = rng.standard_normal((cfg.Hq, 1, k)).astype(np.float32)
    for kvh in range(cfg.Hkv):
        base = int(rng.integers(0, len(cand) - 3 * G))
        for g in range(G):
            picks = [base + g, base + g + 1 + (g % 3)]
            an2[kvh * G + g, 0] = [cand[p][1] for p in picks]
    an2_t, sc2_t = torch.from_numpy(an2).to(DEV), torch.from_numpy(sc2).to(DEV)
    O2 = f64(B.sl_anchor_attention_decode(Q, K, V, an2_t, sc2_t, w, b, f))
    torch.cuda.synchronize()
    for h in list(range(G)) + ([] if name == "C5" else list(range(cfg.Hq - G, cfg.Hq))):   # whole groups
        o = orc.anchor_combined_row(Qn[h, 0], Kd, Vd, h // G, i, w, b, f, an2[h, 0], sc2[h, 0].astype(np.float64),
                                    1.0 / math.sqrt(cfg.D))
        assert float(np.max(np.abs(O2[h, 0] - o))) <= TOL[torch.bfloat16], h


def test_paper_geometry_prefill_all_rows_of_the_256k_cache():
    # the configuration bench.py times: every row of config 4 on the paper's geometry (window 1088,
    # top-2, b = 4, f = 2) through the group-shared search and the bucketed matrix-core attention;
    # sampled rows against the oracle, plus the row-stationary form on a block of rows
    cfg = W.CONFIGS["C4"]
    data = W.generate(cfg, device=DEV)
    Q, K, V = data["Q"], data["K"], data["V"]
    del data
    w, k, b, f = 1088, 2, 4, 2
    G = cfg.Hq // cfg.Hkv
    anchors, sc = B.sl_anchor_search_prefill(Q, K, k, w, want_scores=True)
    O = B.sl_anchor_attention_prefill(Q, K, V, anchors, sc, w, b, f)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()
    rng = np.random.default_rng(3)
    pos = sorted({0, 1, 2, 1087, 1088, 1089, 1152, 5000, cfg.L // 2, cfg.L - 2, cfg.L - 1} |
                 {int(x) for x in rng.integers(0, cfg.L, 24)})
    Kd, Vd = DevKV(K), DevKV(V)
    for h in (0, 9, 31):
        for r in pos:
            qn = f64(Q[h, r])
            an_r, sc_r = anchors[h, r].cpu().numpy(), sc[h, r].cpu().numpy().astype(np.float64)
            _, t_o, _ = orc.anchor_search_row(qn, DevRows(K[h // G]), r, w, k)
            want = t_o + [-1] * (k - len(t_o))
            if an_r.tolist() != want:
                cand = orc.anchor_candidates(r, w)
                allsc = [float(f64(K[h // G, t]) @ qn) for _, t in cand]
                check_anchor_row(an_r.tolist(), want, cand, allsc, k, (h, r))
            sc_r = np.where(np.isfinite(sc_r), sc_r, 0.0)
            o = orc.anchor_combined_row(qn, Kd, Vd, h // G, r, w, b, f, an_r, sc_r, 1.0 / math.sqrt(cfg.D))
            assert float(np.max(np.abs(f64(O[h, r]) - o))) <= TOL[torch.bfloat16], (h, r)
    # a block of rows through the row-stationary kernels
    p0, nr = cfg.L - 3000, 1024
    Or = B.sl_anchor_attention_prefill(Q[:, p0:p0 + nr], K, V, anchors[:, p0:p0 + nr].contiguous(),
                                       sc[:, p0:p0 + nr].contiguous(), w, b, f, q_pos0=p0, row_stationary=True)
    torch.cuda.synchronize()
    assert float((Or.float() - O[:, p0:p0 + nr].float()).abs().max()) <= 1.5 * TOL[torch.bfloat16]
    del K, V
    torch.cuda.empty_cache()
