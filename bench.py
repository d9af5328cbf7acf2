#!/usr/bin/env python3
"""Benchmark of the span-search + span-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--configs C3,C5,...] [--no-cpu-baseline]

A step is one pass of the whole hot path over one batch of synthetic input already resident
in HBM: prefill = span keys + span-search + span-attention over all L queries; decode = span-search
+ span-attention for one new token against the L-token cache (span keys are cache state).
The primary workload (the JSON line's `value`) is the 1M-token decode configuration; the other
four configurations are reported under `all_configs` in the same line.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM = 8.0e12           # B/s, MI355X HBM3E
PEAK_BF16 = 2.5e15          # flop/s, dense bf16 MFMA
PEAK_FP32_VALU = 157.3e12   # flop/s, fp32 vector
N_DECODE_QUERIES = 8        # decode steps rotate over this many independent queries (different span sets)
MAIN_ONLY = False           # --main-only: time only each configuration's own step (clean profiler traces)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class ProfEvents:
    """Two HIP events the library records around its dominant kernel (caller-owned)."""

    def __init__(self, torch):
        self.a = torch.cuda.Event(enable_timing=True)
        self.b = torch.cuda.Event(enable_timing=True)
        self.a.record()
        self.b.record()          # creates the underlying hipEvent_t handles
        torch.cuda.synchronize()

    def handles(self):
        return (self.a.cuda_event, self.b.cuda_event)

    def ms(self):
        self.b.synchronize()
        return self.a.elapsed_time(self.b)


def device_facts(torch):
    """Compute units and maximum clock of GPU 0 as rocminfo reports them (torch's properties as a
    fallback), and the dense bf16 MFMA peak they imply next to the published peaks the roofline uses."""
    import re
    import subprocess
    name, cus, mhz = "", 0, 0.0
    try:
        out = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=30).stdout
        for agent in out.split("*******")[1:]:
            if re.search(r"Device Type:\s+GPU", agent):
                m = re.search(r"Marketing Name:[ \t]*(.*)", agent)
                name = m.group(1).strip() if m else ""
                if not name:                      # some boxes leave the marketing name empty
                    m = re.search(r"^\s*Name:[ \t]*(gfx\w+)", agent, re.M)
                    name = m.group(1) if m else ""
                m = re.search(r"Compute Unit:\s+(\d+)", agent)
                cus = int(m.group(1)) if m else 0
                m = re.search(r"Max Clock Freq\. \(MHz\):\s+(\d+)", agent)
                mhz = float(m.group(1)) if m else 0.0
                break
    except Exception:
        pass
    if not cus:
        prop = torch.cuda.get_device_properties(0)
        name, cus, mhz = prop.name, prop.multi_processor_count, getattr(prop, "clock_rate", 0) / 1e3
    return {"name": name, "compute_units": cus, "max_clock_mhz": mhz,
            # 4 SIMDs x 1024 flop/clk (a 32x32x16 bf16 MFMA = 32768 flop in 32 cycles) per compute unit
            "derived_bf16_mfma_peak_tflops": cus * 4096 * mhz * 1e6 / 1e12,
            "peaks_used": {"hbm_GBps": PEAK_HBM / 1e9, "bf16_mfma_tflops": PEAK_BF16 / 1e12,
                           "fp32_valu_tflops": PEAK_FP32_VALU / 1e12}}


def prefill_flops(cfg):
    """Algorithmic flops of one prefill step: causal search + attention over selected keys."""
    L, S, k, D, Hq = cfg.L, cfg.S, cfg.topk, cfg.D, cfg.Hq
    search = 0
    routed = 0
    local = 0
    for c in range(cfg.n_spans):
        rows = min(S, L - c * S)
        search += rows * c * 2 * D
        # keys per row: min(k, c) * S routed + (i mod S) + 1 in the local window
        routed += rows * min(k, c) * S * 4 * D
        local += rows * (rows + 1) // 2 * 4 * D
    return Hq * search, Hq * routed, Hq * local


TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


def recorded_traffic(name):
    """HBM bytes per launch of a configuration's dominant kernel as recorded by rocprofv3 counter runs
    (FETCH_SIZE + WRITE_SIZE, scaled by the 1 GiB copy calibration): read from the committed table
    under profiles/, which names the kernel and the command of each figure.  None if not recorded."""
    try:
        for line in open(TRAFFIC_TABLE):
            f = line.split()
            if len(f) >= 3 and f[0] == name and not line.startswith("#"):
                return float(f[2])
    except OSError:
        pass
    return None


def decode_bytes(cfg, idx, q_pos):
    """Algorithmic HBM bytes of one decode span-attention: distinct (kv head, span) pairs x K and V rows."""
    G = cfg.Hq // cfg.Hkv
    c = q_pos // cfg.S
    esz = 2 if cfg.dtype == "bf16" else 4
    pairs = set()
    for h, row in enumerate(idx.reshape(cfg.Hq, -1).tolist()):
        for j in row:
            if 0 <= j < c:
                pairs.add((h // G, j))
    tokens = len(pairs) * cfg.S + cfg.Hkv * (q_pos - c * cfg.S + 1)
    return tokens * cfg.D * esz * 2


def bench_decode(cfg, steps, warmup, torch, B, W):
    dev = "cuda"
    data = W.generate(cfg, device=dev, n_queries=N_DECODE_QUERIES)
    K, V = data["K"], data["V"]
    Ks = B.sl_span_keys(K, cfg.S)
    Qs = [data["Q"][i] for i in range(N_DECODE_QUERIES)]
    q_pos = cfg.L - 1
    ws = B.Workspace()
    outs = [(torch.empty((cfg.Hq, 1, cfg.D), dtype=K.dtype, device=dev),
             torch.empty((cfg.Hq, 1), dtype=torch.float32, device=dev)) for _ in range(N_DECODE_QUERIES)]

    def step(i, prof=None):
        q = Qs[i % N_DECODE_QUERIES]
        idx = B.sl_span_search_decode(q, K, Ks, cfg.S, cfg.topk, ws=ws)
        B.sl_span_attention_decode(q, K, V, idx, cfg.S, ws=ws, prof=prof, out=outs[i % N_DECODE_QUERIES])
        return idx

    idxs = [step(i).cpu().numpy() for i in range(N_DECODE_QUERIES)]
    abytes = [decode_bytes(cfg, ix, q_pos) for ix in idxs]
    for i in range(max(warmup, N_DECODE_QUERIES)):
        step(i)
    torch.cuda.synchronize()
    # The decode step is launch-bound on the host (three short kernels), so the timed loop replays
    # a HIP graph that holds N_DECODE_QUERIES consecutive steps (one per rotating query).
    # Exactly `steps` steps are timed: steps // 8 replays of the 8-step graph plus one replay of a graph
    # with the remaining steps.
    steps = max(1, steps)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(N_DECODE_QUERIES):
            step(i)
    rest = steps % N_DECODE_QUERIES
    rgraph = None
    if rest:
        rgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(rgraph):
            for i in range(rest):
                step(i)
        rgraph.replay()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps // N_DECODE_QUERIES):
        graph.replay()
    if rgraph is not None:
        rgraph.replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # per-replay times (HIP events on the launch stream) for the median
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rep_ms = []
    for _ in range(max(3, min(steps // N_DECODE_QUERIES, 25))):
        e0.record()
        graph.replay()
        e1.record()
        e1.synchronize()
        rep_ms.append(e0.elapsed_time(e1) / N_DECODE_QUERIES)
    rep_ms.sort()
    # Dominant kernel, measured next to the timed region (before the variants below allocate their
    # buffers and change what is resident).  K/V streaming + reduce: a graph of N_DECODE_QUERIES back-to-back
    # span-attention launches, timed with HIP events on the launch stream.
    idx_dev = [torch.from_numpy(ix).to(dev) for ix in idxs]
    agraph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(agraph):
        for i in range(N_DECODE_QUERIES):
            B.sl_span_attention_decode(Qs[i], K, V, idx_dev[i], cfg.S, ws=ws, out=outs[i])
    agraph.replay()
    torch.cuda.synchronize()
    entry_ms = []
    for _ in range(max(4, min(steps // N_DECODE_QUERIES, 16))):
        e0.record()
        agraph.replay()
        e1.record()
        e1.synchronize()
        entry_ms.append(e0.elapsed_time(e1) / N_DECODE_QUERIES)
    # ... and the K/V streaming kernel alone, between the two HIP events that the library attaches to
    # its dispatch.  Each timed launch is queued right behind a replay of the step graph, so that
    # the kernel runs at the clocks and cache state of the timed region rather than after an idle gap.
    # Only the first half of the rotating queries is timed: the graph ends with the last one, whose
    # spans may still sit in the 256 MB memory-side cache; a timed query's spans were last read at
    # least N_DECODE_QUERIES / 2 steps (> 1 GB of traffic) earlier.
    evs = [ProfEvents(torch) for _ in range(max(16, min(steps // 4, 48)))]
    for i, ev in enumerate(evs):
        qi = i % (N_DECODE_QUERIES // 2)
        graph.replay()
        B.sl_span_attention_decode(Qs[qi], K, V, idx_dev[qi], cfg.S, ws=ws, out=outs[qi], prof=ev.handles())
    torch.cuda.synchronize()
    kms = [ev.ms() for ev in evs]
    kbytes = abytes[:N_DECODE_QUERIES // 2]
    kms_avg = sum(kms) / len(kms)
    achieved = (sum(kbytes) / len(kbytes)) / (kms_avg * 1e-3)
    dt_combined, paper_geometry, batched = None, None, None
    if not MAIN_ONLY:
        # The combination form of the same steps (search with scores, gated reduction), same replay.
        outs_c = [torch.empty((cfg.Hq, 1, cfg.D), dtype=K.dtype, device=dev) for _ in range(N_DECODE_QUERIES)]

        def step_combined(i):
            q = Qs[i % N_DECODE_QUERIES]
            idx, sc = B.sl_span_search_decode(q, K, Ks, cfg.S, cfg.topk, want_scores=True, ws=ws)
            B.sl_span_attention_combined_decode(q, K, V, idx, sc, cfg.S, ws=ws, out=outs_c[i % N_DECODE_QUERIES])

        for i in range(N_DECODE_QUERIES):
            step_combined(i)
        torch.cuda.synchronize()
        cgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cgraph):
            for i in range(N_DECODE_QUERIES):
                step_combined(i)
        cgraph.replay()
        torch.cuda.synchronize()
        tc = time.perf_counter()
        nrep = max(2, steps // N_DECODE_QUERIES // 2)
        for _ in range(nrep):
            cgraph.replay()
        torch.cuda.synchronize()
        dt_combined = (time.perf_counter() - tc) / (nrep * N_DECODE_QUERIES)
        # The paper's own geometry on the same cache (anchors on the quadratic stride pattern, window
        # 1088, top-2, b = 4, f = 2: Section 4.3's kernel configuration), same replay.
        PW, PK, PB, PF = 1088, 2, 4, 2
        outs_p = [torch.empty((cfg.Hq, 1, cfg.D), dtype=K.dtype, device=dev) for _ in range(N_DECODE_QUERIES)]

        def step_paper(i, prof=None):
            q = Qs[i % N_DECODE_QUERIES]
            an, sc = B.sl_anchor_search_decode(q, K, PK, PW, want_scores=True)
            B.sl_anchor_attention_decode(q, K, V, an, sc, PW, PB, PF, ws=ws, prof=prof, out=outs_p[i % N_DECODE_QUERIES])
            return an

        an0 = [step_paper(i).cpu().numpy() for i in range(N_DECODE_QUERIES)]
        torch.cuda.synchronize()
        pgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(pgraph):
            for i in range(N_DECODE_QUERIES):
                step_paper(i)
        pgraph.replay()
        torch.cuda.synchronize()
        tc = time.perf_counter()
        for _ in range(nrep):
            pgraph.replay()
        torch.cuda.synchronize()
        dt_paper = (time.perf_counter() - tc) / (nrep * N_DECODE_QUERIES)
        # its K/V streaming kernel and algorithmic bytes: per kv head the union of the heads' token
        # ranges (span minus window, plus the window once), K and V rows
        ell = math.isqrt(q_pos) + (0 if math.isqrt(q_pos) ** 2 == q_pos else 1)
        G = cfg.Hq // cfg.Hkv
        pbytes = []
        for an in an0[:N_DECODE_QUERIES // 2]:
            tokens = 0
            for kv in range(cfg.Hkv):
                cover = set()
                for h in range(kv * G, (kv + 1) * G):
                    for t in an[h, 0].tolist():
                        if t >= 0:
                            cover.add((max(0, t - PB * ell), min(min(q_pos, t + PF * ell), q_pos - PW) + 1))
                ivs = sorted(cover)
                end = -1
                for a0, a1 in ivs:          # union of intervals
                    a0 = max(a0, end)
                    if a1 > a0:
                        tokens += a1 - a0
                        end = a1
                tokens += PW
            pbytes.append(tokens * cfg.D * 2 * 2)
        evp = [ProfEvents(torch) for _ in range(16)]
        for i, ev in enumerate(evp):
            qi = i % (N_DECODE_QUERIES // 2)
            pgraph.replay()
            an, sc = B.sl_anchor_search_decode(Qs[qi], K, PK, PW, want_scores=True)
            B.sl_anchor_attention_decode(Qs[qi], K, V, an, sc, PW, PB, PF, ws=ws, prof=ev.handles(), out=outs_p[qi])
        torch.cuda.synchronize()
        pms = sum(ev.ms() for ev in evp) / len(evp)
        paper_geometry = {"workload": f"anchors i-(s+1)^2+1, window {PW}, top-{PK}, b={PB}, f={PF}, combination gate",
                          "ms_per_step": dt_paper * 1e3, "value": 1.0 / dt_paper, "unit": "steps/s",
                          "roofline": {"bound": "hbm", "kernel": "decode_split_kernel", "kernel_ms": pms,
                                       "algorithmic_bytes": sum(pbytes) / len(pbytes),
                                       "achieved": sum(pbytes) / len(pbytes) / (pms * 1e-3) / 1e9,
                                       "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                                       "frac": sum(pbytes) / len(pbytes) / (pms * 1e-3) / PEAK_HBM}}
        # Batched decode: NB sequences with caches of their own (copies of the cache, cut to different
        # lengths, each with a different query) advance one step in three launches.
        esz = 2 if cfg.dtype == "bf16" else 4
        NB = 8 if 8 * 2 * cfg.Hkv * cfg.L * cfg.D * esz <= 64e9 else 4
        lens = [cfg.L - b * (cfg.S + 37) for b in range(NB)]
        Kc = [K.clone()[:, :lens[b]] for b in range(NB)]
        Vc = [V.clone()[:, :lens[b]] for b in range(NB)]
        Ksc = [B.sl_span_keys(Kc[b], cfg.S) for b in range(NB)]
        nrot = max(1, N_DECODE_QUERIES // NB)
        batches = [B.DecodeBatch([Qs[(r * NB + b) % N_DECODE_QUERIES] for b in range(NB)],
                                 [Qs[(r * NB + b) % N_DECODE_QUERIES] for b in range(NB)], Kc, Vc, Ksc,
                                 cfg.S, cfg.topk) for r in range(nrot)]

        def step_batched(r):
            B.sl_span_search_decode_batched(batches[r])
            B.sl_span_attention_decode_batched(batches[r], ws=ws)

        bbytes = 0
        for r in range(nrot):
            step_batched(r)
            torch.cuda.synchronize()
            ix = batches[r].idx.cpu().numpy()
            bbytes += sum(decode_bytes(cfg, ix[b], lens[b] - 1) for b in range(NB))
        bgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(bgraph):
            for r in range(nrot):
                step_batched(r)
        bgraph.replay()
        torch.cuda.synchronize()
        tc = time.perf_counter()
        for _ in range(nrep):
            bgraph.replay()
        torch.cuda.synchronize()
        dt_batched = (time.perf_counter() - tc) / (nrep * nrot)
        batched = {"workload": f"{NB} sequences, caches of {lens[-1]}..{lens[0]} tokens, one query each",
                   "ms_per_step": dt_batched * 1e3, "value": NB / dt_batched, "unit": "sequence-steps/s",
                   "algorithmic_bytes": bbytes / nrot,
                   "step_hbm_frac": bbytes / nrot / dt_batched / PEAK_HBM}
        # ... and the same batch on the paper's geometry (anchors, gated combination)
        pbatch = B.DecodeBatch([Qs[b % N_DECODE_QUERIES] for b in range(NB)], [Qs[b % N_DECODE_QUERIES] for b in range(NB)],
                               Kc, Vc, None, 1, PK, want_scores=True)

        def step_batched_paper():
            B.sl_anchor_search_decode_batched(pbatch, PW)
            B.sl_anchor_attention_decode_batched(pbatch, PW, PB, PF, ws=ws)

        step_batched_paper()
        torch.cuda.synchronize()
        pbgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(pbgraph):
            step_batched_paper()
        pbgraph.replay()
        torch.cuda.synchronize()
        tc = time.perf_counter()
        for _ in range(nrep * 2):
            pbgraph.replay()
        torch.cuda.synchronize()
        dt_bp = (time.perf_counter() - tc) / (nrep * 2)
        batched["paper_geometry"] = {"ms_per_step": dt_bp * 1e3, "value": NB / dt_bp, "unit": "sequence-steps/s"}
        del Kc, Vc, Ksc, batches, bgraph, pbatch, pbgraph
    res = {
        "workload": f"{cfg.name} decode L={cfg.L} Hq={cfg.Hq} Hkv={cfg.Hkv} D={cfg.D} S={cfg.S} topk={cfg.topk}+local",
        "metric": "decode steps/s (span-search + span-attention)", "value": steps / dt, "unit": "steps/s",
        "ms_per_step": dt / steps * 1e3, "ms_per_step_median": rep_ms[len(rep_ms) // 2], "steps": steps,
        "dtype": cfg.dtype, "launch": "hip-graph replay",
        "combined_form": None if dt_combined is None else
        {"ms_per_step": dt_combined * 1e3, "value": 1.0 / dt_combined, "unit": "steps/s"},
        "paper_geometry": paper_geometry,
        "batched_decode": batched,
        "roofline": {"bound": "hbm", "kernel": "decode_split_kernel", "achieved": achieved / 1e9, "peak": PEAK_HBM / 1e9,
                     "unit": "GB/s", "frac": achieved / PEAK_HBM, "traffic": recorded_traffic(cfg.name),
                     "kernel_ms": kms_avg, "kernel_ms_min": min(kms), "algorithmic_bytes": sum(kbytes) / len(kbytes),
                     "attention_entry_ms_graph": sum(entry_ms) / len(entry_ms)},
    }
    return res, dict(data=data, Ks=Ks, idx0=idxs[0])


def bench_prefill(cfg, steps, warmup, torch, B, W):
    dev = "cuda"
    data = W.generate(cfg, device=dev)
    Q, K, V, Qs = data["Q"], data["K"], data["V"], data["Qs"]
    ws = B.Workspace()
    out = (torch.empty((cfg.Hq, cfg.L, cfg.D), dtype=Q.dtype, device=dev),
           torch.empty((cfg.Hq, cfg.L), dtype=torch.float32, device=dev))
    Ks = torch.zeros((cfg.Hkv, cfg.n_spans, cfg.D), dtype=K.dtype, device=dev)

    def step(prof_s=None, prof_a=None):
        B.sl_span_keys(K, cfg.S, out=Ks)
        idx = B.sl_span_search_prefill(Qs, K, Ks, cfg.S, cfg.topk, ws=ws, prof=prof_s)
        B.sl_span_attention_prefill(Q, K, V, idx, cfg.S, ws=ws, prof=prof_a, out=out)
        return idx

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ev_s, ev_a = ProfEvents(torch), ProfEvents(torch)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ms_s, ms_a, step_ms = [], [], []
    for _ in range(max(3, min(steps, 10))):
        e0.record()
        step(ev_s.handles(), ev_a.handles())
        e1.record()
        ms_s.append(ev_s.ms())
        ms_a.append(ev_a.ms())
        e1.synchronize()
        step_ms.append(e0.elapsed_time(e1))
    step_ms.sort()
    dt_combined, chunked, redundant, paper = None, None, None, None
    if not MAIN_ONLY:
        # the combination form (per-span softmaxes gated by the search scores) of the same step
        def step_combined():
            B.sl_span_keys(K, cfg.S, out=Ks)
            idx, sc = B.sl_span_search_prefill(Qs, K, Ks, cfg.S, cfg.topk, want_scores=True, ws=ws)
            B.sl_span_attention_combined_prefill(Q, K, V, idx, sc, cfg.S, ws=ws, out=out[0])

        step_combined()
        torch.cuda.synchronize()
        tc = time.perf_counter()
        nc = max(1, min(steps, 3))
        for _ in range(nc):
            step_combined()
        torch.cuda.synchronize()
        dt_combined = (time.perf_counter() - tc) / nc
        # the same prefill in chunks of 32K query rows against the growing cache (Section 5's chunked
        # prefill): chunk c sees the first (c + 1) * 32K tokens through q_pos0 / Lq
        chunked = None
        CH = 32768
        if cfg.L % CH == 0 and cfg.L > CH:
            och = (torch.empty((cfg.Hq, CH, cfg.D), dtype=Q.dtype, device=dev),
                   torch.empty((cfg.Hq, CH), dtype=torch.float32, device=dev))

            def step_chunked():
                for c in range(cfg.L // CH):
                    p0, vis = c * CH, (c + 1) * CH
                    Kc, Vc = K[:, :vis], V[:, :vis]
                    # span keys are read from the cache itself (no gathered copy per chunk)
                    idx = B.sl_span_search_prefill(Qs[:, p0:vis], Kc, None, cfg.S, cfg.topk, q_pos0=p0, ws=ws)
                    B.sl_span_attention_prefill(Q[:, p0:vis], Kc, Vc, idx, cfg.S, q_pos0=p0, ws=ws, out=och)

            step_chunked()
            torch.cuda.synchronize()
            tch = time.perf_counter()
            nch = max(1, min(steps, 3))
            for _ in range(nch):
                step_chunked()
            torch.cuda.synchronize()
            dt_ch = (time.perf_counter() - tch) / nch
            chunked = {"chunk_rows": CH, "ms_per_step": dt_ch * 1e3, "value": cfg.L / dt_ch, "unit": "tokens/s"}
        # the redundant grid (anchors every S/2 tokens, spans S tokens long: twice the candidates, overlapping
        # spans de-duplicated in the joint softmax) through the same kernels
        redundant = None
        if cfg.dtype == "bf16" and cfg.S % 128 == 0:
            A = cfg.S // 2
            Ks2 = torch.zeros((cfg.Hkv, -(-cfg.L // A), cfg.D), dtype=K.dtype, device=dev)

            def step_redundant():
                B.sl_span_keys(K, A, out=Ks2)
                idx = B.sl_span_search_prefill(Qs, K, Ks2, A, cfg.topk, ws=ws)
                B.sl_span_attention_prefill(Q, K, V, idx, cfg.S, ws=ws, out=out, span_stride=A)

            step_redundant()
            torch.cuda.synchronize()
            tr = time.perf_counter()
            nr = max(1, min(steps, 3))
            for _ in range(nr):
                step_redundant()
            torch.cuda.synchronize()
            dt_r = (time.perf_counter() - tr) / nr
            redundant = {"anchor_spacing": A, "span_length": cfg.S, "topk": cfg.topk, "ms_per_step": dt_r * 1e3,
                         "value": cfg.L / dt_r, "unit": "tokens/s"}
            del Ks2
        # the paper's own geometry in prefill form over ALL rows (every row has its own anchors, span
        # length and window) at the paper's kernel configuration: group-shared anchor search, then the
        # bucketed matrix-core span-attention + banded window + gated merge
        paper = None
        if cfg.dtype == "bf16" and cfg.L >= 16384:
            PW, PK, PB, PF = 1088, 2, 4, 2
            op = out[0]
            ev_p = ProfEvents(torch)

            def step_paper(prof=None):
                an, sc = B.sl_anchor_search_prefill(Qs, K, PK, PW, want_scores=True)
                B.sl_anchor_attention_prefill(Q, K, V, an, sc, PW, PB, PF, out=op, ws=ws, prof=prof)
                return an

            an = step_paper()
            torch.cuda.synchronize()
            tp = time.perf_counter()
            npp = max(1, min(steps, 3))
            for _ in range(npp):
                step_paper(ev_p.handles())
            torch.cuda.synchronize()
            dt_p = (time.perf_counter() - tp) / npp
            kp = ev_p.ms()
            # algorithmic flops of the routed kernel: sum over valid (row, slot) of the span length (span minus window) x 4D
            i_pos = torch.arange(cfg.L, device=dev, dtype=torch.int64)
            ell = torch.sqrt(i_pos.double()).ceil().long()
            ell = torch.where((ell - 1) * (ell - 1) >= i_pos, ell - 1, ell)        # exact ceil(sqrt(i))
            ell = torch.where(ell * ell < i_pos, ell + 1, ell)
            wlo = (i_pos - PW + 1).clamp(min=0)
            keys = 0
            for h0 in range(0, cfg.Hq, 8):
                t = an[h0:h0 + 8].long()                                           # [8, L, k]
                valid = (t >= 0) & (t <= i_pos[None, :, None])
                lo = (t - PB * ell[None, :, None]).clamp(min=0)
                hi = torch.minimum(torch.minimum(t + PF * ell[None, :, None], i_pos[None, :, None]), wlo[None, :, None] - 1) + 1
                keys += int(((hi - lo).clamp(min=0) * valid).sum())
            f_paper = keys * 4 * cfg.D
            paper = {"rows": cfg.L, "window": PW, "topk": PK, "backward_factor": PB, "forward_factor": PF,
                     "ms_per_step": dt_p * 1e3, "value": cfg.L / dt_p, "unit": "tokens/s",
                     "roofline": {"bound": "mfma", "kernel": "span_flash_anchor_kernel", "kernel_ms": kp,
                                  "algorithmic_flops": f_paper, "achieved": f_paper / (kp * 1e-3) / 1e12,
                                  "peak": PEAK_BF16 / 1e12, "unit": "TFLOP/s", "frac": f_paper / (kp * 1e-3) / PEAK_BF16}}
            del an
    f_search, f_routed, f_local = prefill_flops(cfg)
    f_attn = f_routed + f_local
    ka = sum(ms_a) / len(ms_a)
    ks = sum(ms_s) / len(ms_s)
    mfma_path = cfg.dtype == "bf16" and cfg.D == 128 and cfg.S % 64 == 0
    peak, bound = (PEAK_BF16, "mfma") if cfg.dtype == "bf16" else (PEAK_FP32_VALU, "alu")
    # the events bracket the routed-span kernel on the MFMA path, the one attention kernel otherwise
    f_kernel = f_routed if mfma_path else f_attn
    kernel = "span_flash_routed_kernel" if mfma_path else "prefill_attention_rows_kernel"
    tflops_attn = f_kernel / (ka * 1e-3)
    res = {
        "workload": f"{cfg.name} prefill L={cfg.L} Hq={cfg.Hq} Hkv={cfg.Hkv} D={cfg.D} S={cfg.S} topk={cfg.topk}+local",
        "metric": "prefill tokens/s (span-search + span-attention)", "value": cfg.L * steps / dt, "unit": "tokens/s",
        "ms_per_step": dt / steps * 1e3, "ms_per_step_median": step_ms[len(step_ms) // 2], "steps": steps,
        "dtype": cfg.dtype,
        "step_frac_of_peak": (f_search + f_attn) / (dt / steps) / peak,
        "combined_form": None if dt_combined is None else
        {"ms_per_step": dt_combined * 1e3, "value": cfg.L / dt_combined, "unit": "tokens/s"},
        "chunked_prefill": chunked,
        "redundant_spans": redundant,
        "paper_geometry_prefill": paper,
        "roofline": {"bound": bound, "kernel": kernel, "achieved": tflops_attn / 1e12,
                     "peak": peak / 1e12, "unit": "TFLOP/s", "frac": tflops_attn / peak,
                     "traffic": recorded_traffic(cfg.name),
                     "kernel_ms": ka, "algorithmic_flops": f_kernel, "step_algorithmic_flops": f_search + f_attn,
                     "search_kernel_ms": ks, "search_algorithmic_flops": f_search},
    }
    return res, dict(data=data)


def _oracle_threads():
    """Threads the oracle's numpy calls may use; the oracle is plain numpy and is timed on ONE thread."""
    return 1


def cpu_baseline_decode(cfg, ctx, torch, budget_s=6.0):
    """The fp64 oracle, as it stands, on whole decode steps (all heads) of the same workload."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import superlinear as orc

    class HostKV:
        def __init__(self, t):
            self.t = t
            self.shape = t.shape

        def __getitem__(self, key):
            kv, sl = key
            return self.t[kv, sl].float().numpy()

    data, Ks = ctx["data"], ctx["Ks"]
    Kh, Vh = HostKV(data["K"].cpu()), HostKV(data["V"].cpu())
    Ksn = Ks.float().cpu().numpy().astype(np.float64)
    q_pos = cfg.L - 1
    done, t0 = 0, time.perf_counter()
    with threadpool_limits(limits=_oracle_threads()):
        # about budget_s of CPU work: the 8 rotating queries, several times over if they are quick
        while done < 5 * N_DECODE_QUERIES and (time.perf_counter() - t0) < budget_s:
            Qn = data["Q"][done % N_DECODE_QUERIES].float().cpu().numpy().astype(np.float64)
            idx = orc.span_search(Qn, Ksn, cfg.S, cfg.topk, q_pos0=q_pos)
            orc.span_attention(Qn, Kh, Vh, idx, cfg.S, q_pos0=q_pos)
            done += 1
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "steps/s", "cores": _oracle_threads(), "kind": "oracle",
            "sample": f"{done} whole decode steps (all {cfg.Hq} heads, search + attention) of {cfg.name}; "
                      "numpy fp64, BLAS limited to 1 thread, K/V resident in host RAM as bf16"}


def cpu_baseline_prefill(cfg, ctx, torch, budget_s=6.0):
    """The oracle on query positions of the same workload, all heads per position: every position
    when that fits the budget (C1), otherwise a seeded sample that includes the first rows, span
    boundaries and the last row; tokens/s is positions per second (extrapolated when sampled)."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import superlinear as orc
    data = ctx["data"]
    Qh, Kh, Vh = data["Q"].cpu(), data["K"].float().cpu().numpy(), data["V"].float().cpu().numpy()
    Ksn = orc.span_keys(Kh, cfg.S)
    G = cfg.Hq // cfg.Hkv
    S, L = cfg.S, cfg.L
    rng = np.random.default_rng(0)
    special = [0, 1, S - 1, S, S + 1, 2 * S - 1, 2 * S, L - S - 1, L - S, L - 1]
    order = special + rng.choice(L, size=min(L, 2048), replace=False).tolist()
    whole = cfg.L * cfg.Hq <= 20000                 # small enough to do every row
    if whole:
        order = list(range(L))
    rows, t0 = 0, time.perf_counter()
    sc = 1.0 / math.sqrt(cfg.D)
    with threadpool_limits(limits=_oracle_threads()):
        for r in order:
            if not whole and (time.perf_counter() - t0) > budget_s:
                break
            qrow = Qh[:, r].float().numpy().astype(np.float64)
            for h in range(cfg.Hq):
                s_ = orc.search_scores_row(qrow[h], Ksn[h // G], r // S)
                sel = orc.select_topk(s_, cfg.topk)
                orc.attention_row(qrow[h], Kh, Vh, h // G, r, S, sel, sc)
            rows += 1
    dt = time.perf_counter() - t0
    what = f"all {rows} query positions" if whole else \
        f"{rows} positions of the seeded sample (first rows, span boundaries, last rows, random), extrapolated"
    return {"value": rows / dt, "unit": "tokens/s", "cores": _oracle_threads(), "kind": "oracle",
            "sample": f"{what} x all {cfg.Hq} heads of {cfg.name} (search + attention per row); "
                      "numpy fp64, BLAS limited to 1 thread"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--configs", default="C3,C5,C4,C2,C1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--main-only", action="store_true",
                    help="skip the variants timed beside each configuration (gated form, chunked prefill, redundant "
                         "grid, the paper's geometry, batched decode): a profiler trace then holds one workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain elementwise copy of known size (reads 1 GiB, writes 1 GiB) three "
                         "times, so that rocprofv3 FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    global MAIN_ONLY
    MAIN_ONLY = args.main_only
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_18401_amd import binding as B
    from paper_2601_18401_amd import workloads as W
    B.load()    # raises if the HIP library is missing: there is no fallback
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")    # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)       # one kernel: reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    names = [c.strip() for c in args.configs.split(",") if c.strip()]
    results, primary, cpu = {}, None, None
    for name in names:
        cfg = W.CONFIGS[name]
        t_cfg = time.perf_counter()
        if cfg.kind == "decode":
            steps = args.steps
            res, ctx = bench_decode(cfg, steps, args.warmup, torch, B, W)
        else:
            # prefill steps are long: a few of them are enough for a stable mean
            steps = max(2, min(args.steps, 10 if name != "C1" else 50))
            res, ctx = bench_prefill(cfg, steps, min(args.warmup, 2), torch, B, W)
        results[name] = res
        log(f"[bench] {name}: {res['value']:.4g} {res['unit']}, {res['ms_per_step']:.4f} ms/step, "
            f"roofline {res['roofline']['frac'] * 100:.1f}% of {res['roofline']['bound']} "
            f"(kernel {res['roofline']['kernel_ms']:.4f} ms) [{time.perf_counter() - t_cfg:.1f}s]")
        if not args.no_cpu_baseline:
            # the oracle beside every configuration, a bounded sample each (rank 0, one GPU)
            base = (cpu_baseline_decode if cfg.kind == "decode" else cpu_baseline_prefill)(cfg, ctx, torch)
            res["cpu_baseline"] = base
            log(f"[bench] {name} cpu oracle baseline: {base['value']:.4g} {base['unit']} ({base['sample']})")
        if name == names[0]:
            primary = (cfg, res)
            cpu = res.get("cpu_baseline")
        del ctx
        torch.cuda.empty_cache()

    cfg, res = primary
    device = device_facts(torch)
    line = {
        "metric": "span-attn decode steps/s at L=1M" if cfg.name == "C3" else res["metric"],
        "value": res["value"], "unit": res["unit"], "n_gpus": 1, "steps": res["steps"], "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": res["dtype"], "data": "synthetic",
        "config": {"workload": res["workload"], "decode_queries_rotated": N_DECODE_QUERIES},
        "roofline": res["roofline"], "cpu_baseline": cpu,
        "device": device,
        "all_configs": results,
        "context_only": {"paper_whole_model_decode_tokens_per_s_B200": {"1M": 109, "10M": 76}},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
