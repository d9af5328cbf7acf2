// Decode span-attention: split-KV streaming kernel + log-sum-exp reduction.
//
// One query row per head against an L-token cache (Section 4.3, decoding path).  The attended
// set of a head is its <= topk routed spans plus the local window, each a contiguous run of
// K/V rows, so the step is a pure HBM stream: 2 flops per element read.  Work is cut into
// (head, slot, chunk) items of CT tokens so that thousands of workgroups are in flight.
#include <hip/hip_ext.h>

#include <cmath>

#include "kernels.h"
#include "stream_attend.h"

namespace sl {

namespace {

constexpr int kDecodeThreads = 256;

// Span extents of the paper's geometry for one decode step (l = ceil(i^(1-p)): back = b*l, fwd = f*l).
struct AnchorRanges {
  bool on;
  int64_t wlo, back, fwd;
  int wchunks;  // chunks of the window (it is shorter than the spans: fewer items, fewer records)
};

// Partial record of one (head, slot, chunk): o[D] (unnormalised, relative to m), m (log2 units), l.
// U: 16-byte K loads (and as many V loads) in flight per lane.
// AG: the paper's geometry (ar describes it) instead of the span grid.
template <typename T, int D, int U, bool AG>
__device__ __forceinline__ void decode_split_body(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ idx, float* __restrict__ part, int64_t q_pos, int Hq, int Hkv,
    int S, int A, bool clip, int topk, int nchunks, int CT, float scale_log2e, int64_t qsh, int64_t kvsh,
    int64_t kvst, int n_routed_blocks, int local_stride, bool share_window, const AnchorRanges ar) {
  // Grid: anchors every A tokens, span j = the S tokens ending at (j+1)*A - 1 (A = S: disjoint spans).
  // clip (joint softmax with A < S): spans of one head overlap, and a token must count once, so an
  // entry's range starts behind the end of the nearest lower span that the same head lists.
  // AG: the paper's geometry (Section 3.3, Algorithm 1) instead of the grid: idx holds anchor
  // tokens, slot s of head h attends S_t minus W for t = idx[h][s] (W is a suffix of [0, q_pos], so
  // the set difference is a clip; DedupConcat(S_t, W) is then the slot's range plus the window's),
  // S_t = [max(0, t - back), min(q_pos, t + fwd)], and slot topk of every head is W = [wlo, q_pos].
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  constexpr int NG = (kDecodeThreads / 64) * RPW;  // row groups per workgroup
  __shared__ float s_m[NG], s_l[NG];
  __shared__ float s_o[NG][D];

  const int G = Hq / Hkv;
  const int64_t c = q_pos / A;
  int h, slot, ck;
  // The local-window items come first in the grid: they are served by the L2 after their first
  // reader, and at the end of the grid they would leave the HBM idle while the last of them run.
  const int n_local_blocks = (int)gridDim.x - n_routed_blocks;
  int bid = (int)blockIdx.x - n_local_blocks;
  if (AG) {
    // the paper's geometry: the window is slot topk of every head, Hq * wchunks items, again at
    // the front of the grid (a window item that serves its whole group runs the longest)
    const int b = (int)blockIdx.x, nwin = Hq * ar.wchunks;
    if (b < nwin) {
      h = b / ar.wchunks;
      ck = b % ar.wchunks;
      slot = topk;
    } else {
      ck = (b - nwin) % nchunks;
      const int u = (b - nwin) / nchunks;
      h = u / topk;
      slot = u % topk;
    }
  } else if (bid >= 0) {
    ck = bid % nchunks;
    const int u = bid / nchunks;
    h = u / topk;
    slot = u % topk;
  } else {
    // The G heads of one kv head read the same rows; their block ids differ by a multiple of 8
    // so that they run on the same XCD and share its L2.
    const int lid = (int)blockIdx.x;
    const int hl = lid / local_stride, r = lid % local_stride;
    if (r >= Hkv * nchunks) return;
    const int kv = r / nchunks;
    ck = r % nchunks;
    h = kv * G + hl;
    slot = topk;
  }
  const int kv = h / G;

  // chunk ck of span j as head hh attends it: [t0, t1), empty for an empty slot or past the range
  auto grid_chunk = [&](int hh, int64_t j, int64_t& t0, int64_t& t1) {
    t0 = t1 = 0;
    if (j < 0 || j >= c) return;
    const int64_t end = (j + 1) * A;
    int64_t begin = end - S > 0 ? end - S : 0;
    if (clip) {
      for (int s2 = 0; s2 < topk; ++s2) {
        const int64_t jj = idx[(int64_t)hh * topk + s2];
        if (jj >= 0 && jj < j && (jj + 1) * A > begin) begin = (jj + 1) * A;
      }
    }
    t0 = begin + (int64_t)ck * CT;
    t1 = t0 + CT < end ? t0 + CT : end;
    if (t1 < t0) t1 = t0;
  };
  // The paper's geometry: tokens [r0, r1) that the anchor token t contributes (S_t minus the window).
  auto anchor_range = [&](int64_t t, int64_t& r0, int64_t& r1) {
    r0 = r1 = 0;
    if (t < 0 || t > q_pos) return;
    r0 = t - ar.back > 0 ? t - ar.back : 0;
    const int64_t e = t + ar.fwd < q_pos ? t + ar.fwd : q_pos;
    r1 = (e < ar.wlo - 1 ? e : ar.wlo - 1) + 1;
    if (r1 < r0) r1 = r0;
  };
  // [t0, t1): the tokens of this item.  cb: where the item's CT-token chunk starts (the wavefronts
  // split the chunk from there).  On the grid a chunk starts at a multiple of CT behind the span's
  // first token; on the paper's geometry, where spans of different heads overlap at any offset,
  // chunks sit on the absolute CT-token lattice (chunk number a), so that overlapping spans are cut
  // into the same pieces and a piece can be read once for all of them; a range then touches at
  // most ceil(length / CT) + 1 chunks, which is what nchunks counts in that mode.
  int64_t t0, t1, cb, a_chunk = 0;
  if (AG) {
    int64_t r0, r1;
    if (slot == topk) {
      r0 = ar.wlo;
      r1 = q_pos + 1;
    } else {
      anchor_range(idx[(int64_t)h * topk + slot], r0, r1);
    }
    a_chunk = r0 / CT + ck;
    cb = a_chunk * CT;
    t0 = r0 > cb ? r0 : cb;
    t1 = r1 < cb + CT ? r1 : cb + CT;
    if (t1 < t0) t1 = t0;
  } else if (slot < topk) {
    grid_chunk(h, idx[(int64_t)h * topk + slot], t0, t1);
    cb = t0;
  } else {
    t0 = c * A + (int64_t)ck * CT;
    t1 = t0 + CT < q_pos + 1 ? t0 + CT : q_pos + 1;
    cb = t0;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  // each wave takes a contiguous quarter of the chunk; one batch of loads covers it when it is
  // at most RPW * U rows long
  const int per_wave = CT / (kDecodeThreads / 64);
  const bool one_batch = U <= 8 && per_wave <= RPW * U;  // (wide batches go with chunks of several batches)

  // Rows that several heads of a kv head attend are read once.  (1) Grid: a span that several
  // heads select; paper's geometry: a chunk that the spans of several (head, slot) entries cover
  // (equal anchors, or merely overlapping spans).  The entry that comes first in the group's index
  // rows owns the chunk and computes the partial of every other entry that attends it; the
  // workgroups of those entries leave at once.  Needs the group's G * topk indices in one pass of
  // a wavefront (larger groups: every entry reads its own rows).  (2) share_window: the local
  // window, which all G heads attend: the first head's workgroup serves the group.  When the
  // wave's rows fit one batch they stay in registers and every entry is computed from them;
  // otherwise (and for clipped overlapping grid spans, whose range differs per entry) the owner
  // reads the rows again per entry, through the L2.
  constexpr int kShareWords = 4;  // up to 256 (head, slot) entries per kv head
  const bool dedup = slot < topk && G * topk <= 64 * kShareWords && G > 1;
  const bool window_group = slot == topk && share_window && one_batch && G > 1 && G <= 64;
  unsigned long long share[kShareWords] = {0ull, 0ull, 0ull, 0ull};
  // entry numbers: (head in group) * topk + slot for a span, head in group for the window
  const int my_entry = window_group ? h - kv * G : (h - kv * G) * topk + slot;
  bool multi = false;
  if (dedup && (!AG || t0 < t1)) {
    // every wavefront builds the masks by itself (no LDS, no barrier): lane l looks at entries
    // l, l + 64, ... of the group's index rows, which are contiguous
    const int64_t jmine = idx[(int64_t)h * topk + slot];
    int first = -1, count = 0;
#pragma unroll
    for (int w = kShareWords - 1; w >= 0; --w) {
      const int e = 64 * w + lane;
      int64_t jother = -1;
      if (e < G * topk) jother = idx[(int64_t)kv * G * topk + e];
      bool same;
      if (AG) {  // the other entry's span reaches into this chunk
        int64_t e0, e1;
        anchor_range(jother, e0, e1);
        same = e1 > e0 && e0 < cb + CT && e1 > cb;
      } else {
        same = jmine >= 0 && jmine < c && jother == jmine;
      }
      share[w] = __ballot(same);
      if (share[w]) first = 64 * w + __builtin_ctzll(share[w]);
      count += __builtin_popcountll(share[w]);
    }
    if (count > 1) {
      if (first != my_entry) return;  // the owner writes this entry's record
      multi = true;
    }
  } else if (window_group) {
    if (my_entry != 0) return;
    share[0] = G == 64 ? ~0ull : (1ull << G) - 1ull;
    multi = true;
  }
  const bool per_entry_range = multi && !window_group && clip && !AG;
  const bool from_regs = multi && one_batch && !per_entry_range;

  const int g = lane / LPR, lr = lane % LPR;
  const T* Kb = K + (int64_t)kv * kvsh;
  const T* Vb = V + (int64_t)kv * kvsh;
  const int gi = wave * RPW + g;

  // Merges the workgroup's NG row-group states through the LDS and writes the record.
  auto merge_and_write = [&](const AttendState<T, D>& st, float* prec) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) s_o[gi][lr * EPL + e] = st.o[e];
    if (lr == 0) {
      s_m[gi] = st.m;
      s_l[gi] = st.l;
    }
    __syncthreads();
    if (tid < D) {
      float M = -INFINITY;
#pragma unroll
      for (int i = 0; i < NG; ++i) M = fmaxf(M, s_m[i]);
      float acc = 0.f, lt = 0.f;
#pragma unroll
      for (int i = 0; i < NG; ++i) {
        const float mi = s_m[i];
        if (mi > -INFINITY) {
          const float w = fast_exp2(mi - M);
          acc = fmaf(w, s_o[i][tid], acc);
          lt = fmaf(w, s_l[i], lt);
        }
      }
      prec[tid] = acc;
      if (tid == 0) {
        prec[D] = M;
        prec[D + 1] = lt;
      }
    }
  };
  auto write_empty = [&](float* prec) {
    if (tid < D) prec[tid] = 0.f;
    if (tid == 0) {
      prec[D] = -INFINITY;
      prec[D + 1] = 0.f;
    }
  };
  auto scaled_query = [&](const uint4& raw, float (&q2)[EPL]) {
    float qf[EPL];
    Elem<T>::unpack(raw, qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) q2[e] = qf[e] * scale_log2e;
  };
  // entry -> (head, slot) of the record
  auto entry_head = [&](int e) { return window_group ? kv * G + e : kv * G + e / topk; };
  auto entry_slot = [&](int e) { return window_group ? topk : e % topk; };
  // takes `entry` out of the masks and returns the next entry that attends the same rows, or -1
  // (all threads hold the same masks)
  auto next_entry = [&](int entry) {
    int next = -1;
#pragma unroll
    for (int w = kShareWords - 1; w >= 0; --w) {
      if (w == (entry >> 6)) share[w] &= ~(1ull << (entry & 63));
      if (share[w]) next = 64 * w + __builtin_ctzll(share[w]);
    }
    return next;
  };
  // An entry's share of the chunk and its record.  Grid, window: the item's own [t0, t1) and
  // chunk number.  Paper's geometry: the entry's span cut to the lattice chunk, and the chunk's
  // number counted from the span's own first chunk.
  auto entry_piece = [&](int he, int se, int64_t anchor, int64_t& lo, int64_t& hi) -> float* {
    int cke = ck;
    lo = t0;
    hi = t1;
    if (AG && se < topk) {
      int64_t e0, e1;
      anchor_range(anchor, e0, e1);
      lo = e0 > cb ? e0 : cb;
      hi = e1 < cb + CT ? e1 : cb + CT;
      if (hi < lo) hi = lo;
      cke = (int)(a_chunk - e0 / CT);
    }
    return part + (((int64_t)he * (topk + 1) + se) * nchunks + cke) * (D + 2);
  };
  // the wavefront's rows of the chunk
  const int64_t w0 = cb + (int64_t)wave * per_wave;
  const int64_t cend = AG ? (cb + CT < q_pos + 1 ? cb + CT : q_pos + 1) : t1;  // last row that may be loaded, + 1
  const int64_t w1 = w0 + per_wave < cend ? w0 + per_wave : cend;

  if (U <= 8 && from_regs) {
    // several entries, one chunk, one batch: the rows are loaded once and stay in registers
    if (t0 >= t1) {  // (the window past its end: the same for every head)
      for (int entry = my_entry; entry >= 0; entry = next_entry(entry))
        write_empty(part + (((int64_t)entry_head(entry) * (topk + 1) + entry_slot(entry)) * nchunks + ck) * (D + 2));
      return;
    }
    uint4 kr[U], vr[U];
    uint4 qraw = load16(Q + (int64_t)h * qsh + lr * EPL);
    int64_t anchor = slot < topk ? idx[(int64_t)h * topk + slot] : -1;
    load_rows<T, D, U, true>(Kb, Vb, kvst, w0, w1, lane, kr, vr);
    int entry = my_entry;
    while (true) {
      const int next = next_entry(entry);
      float q2[EPL];
      scaled_query(qraw, q2);
      // the next entry's query (and anchor) are fetched while this one is computed
      int64_t anchor_next = -1;
      if (next >= 0) {
        qraw = load16(Q + (int64_t)entry_head(next) * qsh + lr * EPL);
        if (!window_group) anchor_next = idx[(int64_t)kv * G * topk + next];
      }
      int64_t lo, hi;
      float* prec = entry_piece(entry_head(entry), entry_slot(entry), anchor, lo, hi);
      AttendState<T, D> st;
      st.init();
      // (the rows stay packed between entries: without this the compiler unpacks all of them to
      // fp32 ahead of the loop, which takes twice the registers)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        asm volatile("" : "+v"(kr[u].x), "+v"(kr[u].y), "+v"(kr[u].z), "+v"(kr[u].w));
        asm volatile("" : "+v"(vr[u].x), "+v"(vr[u].y), "+v"(vr[u].z), "+v"(vr[u].w));
      }
      // (positions as offsets from the chunk's first row: they fit 32 bits; the wavefront's share of
      // the chunk may be shorter than the batch)
      const int hi_rel = (int)(hi - cb), wave_end = (wave + 1) * per_wave;
      attend_loaded<T, D, U>(q2, kr, vr, wave * per_wave, (int)(lo - cb), hi_rel < wave_end ? hi_rel : wave_end,
                             lane, st);
      merge_and_write(st, prec);
      if (next < 0) break;
      entry = next;
      anchor = anchor_next;
      __syncthreads();  // the merge above has read s_o / s_m / s_l
    }
    return;
  }

  // One entry, or several whose rows are read again per entry (through the L2).
  int entry = my_entry;
  while (true) {
    const int he = multi ? entry_head(entry) : h;
    const int se = multi ? entry_slot(entry) : slot;
    if (per_entry_range) {  // the entry's own clip
      grid_chunk(he, idx[(int64_t)he * topk + se], t0, t1);
      cb = t0;
    }
    int64_t lo, hi;
    float* prec = entry_piece(he, se, se < topk ? (int64_t)idx[(int64_t)he * topk + se] : (int64_t)-1, lo, hi);
    if (lo >= hi) {  // empty slot or chunk past the end of the range (uniform over the workgroup)
      write_empty(prec);
    } else {
      float q2[EPL];
      scaled_query(load16(Q + (int64_t)he * qsh + lr * EPL), q2);
      // the wavefront's rows of the chunk, cut to the entry's piece
      int64_t v0 = cb + (int64_t)wave * per_wave, v1 = v0 + per_wave;
      v0 = v0 > lo ? v0 : lo;
      v1 = v1 < hi ? v1 : hi;
      AttendState<T, D> st;
      st.init();
      // Rows that one entry reads are streamed past the caches; the window (read by all G heads
      // of its kv head) and shared rows (read again right away) stay cacheable.
      if (slot != topk && !multi)
        attend_range<T, D, U, true>(q2, Kb, Vb, kvst, v0, v1, lane, st);
      else
        attend_range<T, D, U, false>(q2, Kb, Vb, kvst, v0, v1, lane, st);
      merge_and_write(st, prec);
    }
    if (!multi) break;
    const int next = next_entry(entry);
    if (next < 0) break;
    entry = next;
    __syncthreads();  // the merge above has read s_o / s_m / s_l
  }
}

// Registers: the narrow-batch kernels are held to four wavefronts per SIMD (128 registers), which
// they need without the multi-entry loop; left alone, the compiler keeps the loop's unpacked rows
// in registers and halves the occupancy of every workgroup for the sake of a few.
template <typename T, int D, int U, bool AG>
__global__ __launch_bounds__(kDecodeThreads) __attribute__((amdgpu_waves_per_eu(U <= 8 ? 4 : 2)))
void decode_split_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ idx, float* __restrict__ part, int64_t q_pos, int Hq, int Hkv,
    int S, int A, bool clip, int topk, int nchunks, int CT, float scale_log2e, int64_t qsh, int64_t kvsh,
    int64_t kvst, int n_routed_blocks, int local_stride, bool share_window, const AnchorRanges ar) {
  decode_split_body<T, D, U, AG>(Q, K, V, idx, part, q_pos, Hq, Hkv, S, A, clip, topk, nchunks, CT, scale_log2e,
                          qsh, kvsh, kvst, n_routed_blocks, local_stride, share_window, ar);
}

// Batched decode: blockIdx.y is the sequence; its tensors and length come from the device array.
// kvsh = 0: the cache of every sequence is packed for its own length.
// The paper's geometry for a batch: window, span factors and exponent are common, the span base
// length l(L - 1) and the window's first token follow from each sequence's own length.
struct AnchorBatch {
  bool on;
  int64_t window;
  int b, f, root;
  int wchunks;
};

// (the paper's geometry for a batch carries each sequence's own span extents on top: three
// wavefronts per SIMD there, rather than spills)
template <typename T, int D, int U, bool AG>
__global__ __launch_bounds__(kDecodeThreads) __attribute__((amdgpu_waves_per_eu(U <= 8 ? (AG ? 3 : 4) : 2)))
void decode_split_batched_kernel(
    const sl_decode_seq* __restrict__ seqs, float* __restrict__ part, int64_t part_stride, int Hq,
    int Hkv, int S, int A, bool clip, int topk, int nchunks, int CT, float scale_log2e, int64_t qsh,
    int64_t kvsh, int64_t kvst, int n_routed_blocks, int local_stride, bool share_window,
    const AnchorBatch ab) {
  const sl_decode_seq sq = seqs[blockIdx.y];
  const int64_t i = sq.L - 1;
  AnchorRanges ar{false, 0, 0, 0, 0};
  if (AG) {
    const int64_t ell = span_base_length(i, ab.root);
    ar.on = true;
    ar.wlo = ab.window > 0 ? (i - ab.window + 1 > 0 ? i - ab.window + 1 : 0) : i + 1;
    ar.back = (int64_t)ab.b * ell;
    ar.fwd = (int64_t)ab.f * ell;
    ar.wchunks = ab.wchunks;
  }
  decode_split_body<T, D, U, AG>(static_cast<const T*>(sq.Q), static_cast<const T*>(sq.K),
                          static_cast<const T*>(sq.V), sq.idx, part + blockIdx.y * part_stride, i, Hq,
                          Hkv, S, A, clip, topk, nchunks, CT, scale_log2e, qsh, kvsh ? kvsh : sq.L * kvst,
                          kvst, n_routed_blocks, local_stride, share_window, ar);
}

// Merges the (topk + 1) * nchunks partial records of a head.  grid (Hq, D / 32): each workgroup
// produces 32 output dims; its 256 threads are 8 record subsets x 32 dims.  All record loads of a
// thread are issued before the first dependent use, so the kernel costs about two memory round
// trips (statistics, then the partial outputs) instead of one per record.
constexpr int kReduceDims = 32;
constexpr int kReduceSub = 256 / kReduceDims;
constexpr int kReduceBatch = 16;  // records per thread held in registers at a time

template <typename T, int D>
__device__ __forceinline__ void decode_reduce_body(const float* __restrict__ part, T* __restrict__ O,
                                                   float* __restrict__ LSE, int nrec) {
  extern __shared__ float s_w[];  // nrec weights
  __shared__ float s_red[4];
  __shared__ float s_acc[256];
  const int h = blockIdx.x, d0 = blockIdx.y * kReduceDims;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* base = part + (int64_t)h * nrec * (D + 2);
  const int d = tid % kReduceDims, sub = tid / kReduceDims;

  // first batch of partial outputs: independent of the statistics, issued first
  float ov[kReduceBatch];
#pragma unroll
  for (int i = 0; i < kReduceBatch; ++i) {
    const int p = sub + i * kReduceSub;
    ov[i] = p < nrec ? base[(int64_t)p * (D + 2) + d0 + d] : 0.f;
  }

  float M = -INFINITY;
  for (int p = tid; p < nrec; p += 256) {
    const float mp = base[(int64_t)p * (D + 2) + D];
    s_w[p] = mp;
    M = fmaxf(M, mp);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
  if (lane == 0) s_red[wave] = M;
  __syncthreads();
  M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  __syncthreads();

  float lt = 0.f;
  for (int p = tid; p < nrec; p += 256) {
    const float mp = s_w[p];
    const float w = mp > -INFINITY ? fast_exp2(mp - M) : 0.f;
    s_w[p] = w;
    if (w > 0.f) lt = fmaf(w, base[(int64_t)p * (D + 2) + D + 1], lt);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) lt += __shfl_xor(lt, off, 64);
  if (lane == 0) s_red[wave] = lt;
  __syncthreads();
  lt = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);

  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < kReduceBatch; ++i) {
    const int p = sub + i * kReduceSub;
    if (p < nrec) {
      const float w = s_w[p];
      acc = w > 0.f ? fmaf(w, ov[i], acc) : acc;
    }
  }
  for (int p0 = kReduceBatch * kReduceSub; p0 < nrec; p0 += kReduceBatch * kReduceSub) {
#pragma unroll
    for (int i = 0; i < kReduceBatch; ++i) {
      const int p = p0 + sub + i * kReduceSub;
      ov[i] = p < nrec ? base[(int64_t)p * (D + 2) + d0 + d] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kReduceBatch; ++i) {
      const int p = p0 + sub + i * kReduceSub;
      if (p < nrec) {
        const float w = s_w[p];
        acc = w > 0.f ? fmaf(w, ov[i], acc) : acc;
      }
    }
  }
  s_acc[tid] = acc;
  __syncthreads();
  if (tid < kReduceDims) {
    float tot = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < kReduceSub; ++s2) tot += s_acc[s2 * kReduceDims + tid];
    Elem<T>::store1(O + (int64_t)h * D + d0 + tid, tot / lt);
    if (tid == 0 && blockIdx.y == 0) LSE[h] = (M + __log2f(lt)) * kLn2;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_reduce_kernel(const float* __restrict__ part,
                                                            T* __restrict__ O,
                                                            float* __restrict__ LSE, int nrec) {
  decode_reduce_body<T, D>(part, O, LSE, nrec);
}

// Batched decode: blockIdx.z is the sequence.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_reduce_batched_kernel(
    const sl_decode_seq* __restrict__ seqs, const float* __restrict__ part, int64_t part_stride, int nrec) {
  const sl_decode_seq sq = seqs[blockIdx.z];
  decode_reduce_body<T, D>(part + blockIdx.z * part_stride, static_cast<T*>(sq.O), sq.LSE, nrec);
}


// Combination form of the reduction (Section 3.4, eq. (5)-(6); Algorithm 1) for one query: per
// valid slot t, A_t = merge of the slot's chunk records with the window's chunk records (its own
// softmax over span t and the window); O = sum_t alpha_t A_t, alpha = softmax of the slots' search
// scores; no valid slot: the window alone.  Record p = slot * nchunks + chunk (slot topk = window)
// holds (o[D] unnormalised, m, l), m in log2 units; a slot without a span has m = -inf in all
// its records.  grid (Hq, D / 32) like decode_reduce_kernel: 256 threads = 8 chunk subsets x 32
// dims.
constexpr int kMaxSlots = SL_MAX_TOPK + 1;

template <typename T, int D>
__device__ __forceinline__ void decode_reduce_combined_body(const float* __restrict__ part,
                                                            const float* __restrict__ gate,
                                                            T* __restrict__ O, int topk, int nchunks,
                                                            int wchunks) {
  extern __shared__ float s_dyn[];  // [nrec] m, then each record's weight inside its slot; [nrec] l
  __shared__ float s_ms[kMaxSlots], s_ls[kMaxSlots];           // per slot: max m, l relative to it
  __shared__ float s_gate[kMaxSlots];
  __shared__ float s_part[kMaxSlots][kReduceSub][kReduceDims];  // per slot and subset: o relative to it
  const int h = blockIdx.x, d0 = blockIdx.y * kReduceDims;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int d = tid % kReduceDims, sub = tid / kReduceDims;
  const int nslot = topk + 1, nrec = nslot * nchunks;
  // the window (last slot) has only wchunks <= nchunks records; the rest of its row was never written
  const int nvalid = topk * nchunks + wchunks;
  float* s_m = s_dyn;
  float* s_l = s_dyn + nrec;
  const float* base = part + (int64_t)h * nrec * (D + 2);

  // Every global load of the kernel is issued before the first wait: the gate, the partial outputs
  // (a thread owns dim d and the chunks sub, sub + 8, ... of every slot; if they fit kMaxPre
  // registers) and the statistics.  The kernel then costs one memory round trip.
  const float gate_mine = tid < topk ? gate[(int64_t)h * topk + tid] : 0.f;
  constexpr int kMaxPre = 36;
  const int per_slot = (nchunks + kReduceSub - 1) / kReduceSub;
  const int nload = nslot * per_slot;
  const bool pre = nload <= kMaxPre;
  float ov[kMaxPre];
  if (pre) {
    int slot = 0, it = 0;
#pragma unroll
    for (int u = 0; u < kMaxPre; ++u) {
      const int ck = sub + it * kReduceSub;
      ov[u] = (u < nload && ck < nchunks && slot * nchunks + ck < nvalid)
                  ? base[(int64_t)(slot * nchunks + ck) * (D + 2) + d0 + d]
                  : 0.f;
      if (++it == per_slot) {
        it = 0;
        ++slot;
      }
    }
  }
  for (int p = tid; p < nrec; p += 256) {
    s_m[p] = p < nvalid ? base[(int64_t)p * (D + 2) + D] : -INFINITY;
    s_l[p] = p < nvalid ? base[(int64_t)p * (D + 2) + D + 1] : 0.f;
  }
  if (tid < topk) s_gate[tid] = gate_mine;
  __syncthreads();
  // Per slot: the maximum of its records' m, its l relative to that, and each record's weight
  // 2^(m_p - max) (written over m_p).  A wavefront takes slots wave, wave + 4, ...; its lanes
  // stride over the chunks.  (LDS operations of one wavefront complete in issue order.)
  for (int slot = wave; slot < nslot; slot += 4) {
    float m = -INFINITY;
    for (int ck = lane; ck < nchunks; ck += 64) m = fmaxf(m, s_m[slot * nchunks + ck]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    float l = 0.f;
    for (int ck = lane; ck < nchunks; ck += 64) {
      const float mp = s_m[slot * nchunks + ck];
      const float w = mp > -INFINITY ? fast_exp2(mp - m) : 0.f;
      s_m[slot * nchunks + ck] = w;
      l = fmaf(w, s_l[slot * nchunks + ck], l);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) l += __shfl_xor(l, off, 64);
    if (lane == 0) {
      s_ms[slot] = m;
      s_ls[slot] = l;
    }
  }
  __syncthreads();
  if (pre) {
    int slot = 0, it = 0;
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < kMaxPre; ++u) {
      if (u < nload) {
        const int ck = sub + it * kReduceSub;
        if (ck < nchunks) {
          const float w = s_m[slot * nchunks + ck];
          acc = w > 0.f ? fmaf(w, ov[u], acc) : acc;  // (a record without tokens may hold anything)
        }
        if (++it == per_slot) {
          s_part[slot][sub][d] = acc;
          acc = 0.f;
          it = 0;
          ++slot;
        }
      }
    }
  } else {
    for (int slot = 0; slot < nslot; ++slot) {
      float acc = 0.f;
      for (int ck = sub; ck < nchunks; ck += kReduceSub) {
        const float w = s_m[slot * nchunks + ck];
        if (w > 0.f) acc = fmaf(w, base[(int64_t)(slot * nchunks + ck) * (D + 2) + d0 + d], acc);
      }
      s_part[slot][sub][d] = acc;
    }
  }
  __syncthreads();
  // The gated sum over the slots, eight slots at a time (thread = dim d, slots sub, sub + 8, ...).
  auto slot_o = [&](int slot) {
    float o = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < kReduceSub; ++s2) o += s_part[slot][s2][d];
    return o;
  };
  float gmax = (lane < topk && s_ms[lane] > -INFINITY) ? s_gate[lane] : -INFINITY;  // topk <= 32 < 64
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) gmax = fmaxf(gmax, __shfl_xor(gmax, off, 64));
  const float mw = s_ms[topk], lw = s_ls[topk];  // the window always holds the query's own token
  const float ow = slot_o(topk);
  float acc = 0.f, asum = 0.f;
  for (int slot = sub; slot < topk; slot += kReduceSub) {
    const float m = s_ms[slot];
    if (m == -INFINITY) continue;
    const float M = fmaxf(m, mw);
    const float wa = fast_exp2(m - M), wb = fast_exp2(mw - M);
    const float a = __expf(s_gate[slot] - gmax);
    asum += a;
    acc = fmaf(a, (slot_o(slot) * wa + ow * wb) / (s_ls[slot] * wa + lw * wb), acc);
  }
  __shared__ float s_acc[kReduceSub][kReduceDims], s_asum[kReduceSub];
  s_acc[sub][d] = acc;
  if (d == 0) s_asum[sub] = asum;
  __syncthreads();
  if (tid < kReduceDims) {
    float at = 0.f, st = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < kReduceSub; ++s2) {
      at += s_acc[s2][tid];
      st += s_asum[s2];
    }
    Elem<T>::store1(O + (int64_t)h * D + d0 + tid, st > 0.f ? at / st : (lw > 0.f ? ow / lw : 0.f));
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_reduce_combined_kernel(const float* __restrict__ part,
                                                                    const float* __restrict__ gate,
                                                                    T* __restrict__ O, int topk,
                                                                    int nchunks, int wchunks) {
  decode_reduce_combined_body<T, D>(part, gate, O, topk, nchunks, wchunks);
}

// Batched decode: blockIdx.z is the sequence; the gate is the sequence's own score array.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_reduce_combined_batched_kernel(
    const sl_decode_seq* __restrict__ seqs, const float* __restrict__ part, int64_t part_stride, int topk,
    int nchunks, int wchunks) {
  const sl_decode_seq sq = seqs[blockIdx.z];
  decode_reduce_combined_body<T, D>(part + blockIdx.z * part_stride, sq.scores, static_cast<T*>(sq.O), topk,
                                    nchunks, wchunks);
}

// Loads in flight per lane: a wavefront's quarter of a 512-token chunk is two batches of 16 K and
// 16 V loads (measured 4.5 % faster than four batches of 8 at the 10M cache); shorter chunks keep
// 8, which covers a 128-token chunk's quarter in one batch and leaves registers for a fifth
// wavefront per SIMD.
inline bool wide_batches(int CT) { return CT >= 512; }

// One workgroup serving the window of all G heads of a kv head computes them one after the other,
// about a microsecond per head; that pays (fewer workgroups, the rows pulled once) only while the
// rest of the grid runs much longer: from 128 MB of routed K/V rows, about 20 us of streaming.
inline bool window_by_one_workgroup(int64_t routed_items, int CT, int D, size_t elem_bytes) {
  return routed_items * CT * 2 * D * (int64_t)elem_bytes >= ((int64_t)128 << 20);
}

template <typename T, int D, int U, bool AG>
void launch_split_u(int grid, hipStream_t st, hipEvent_t e0, hipEvent_t e1, const void* Q, const void* K,
                    const void* V, const int32_t* idx, float* part, const Problem& pb, int S, int nchunks,
                    int CT, int n_routed, int local_stride, const AnchorRanges& ar) {
  const float scale_log2e = pb.scale * kLog2e;
  const bool clip = !AG && pb.A < pb.S && !pb.combined;  // overlapping spans in one joint softmax
  const bool share_window = window_by_one_workgroup(n_routed, CT, D, sizeof(T));
  if (e0) {
    // With profiling events the launch itself carries them: they then hold the kernel's own
    // begin and end timestamps (events recorded on the stream before / after a 45 us kernel would
    // add the dispatch gaps, several microseconds).
    hipExtLaunchKernelGGL((decode_split_kernel<T, D, U, AG>), dim3(grid), dim3(kDecodeThreads), 0, st, e0, e1,
                          0, static_cast<const T*>(Q), static_cast<const T*>(K),
                          static_cast<const T*>(V), idx, part, pb.q_pos0, pb.Hq, pb.Hkv, S, AG ? S : pb.A,
                          clip, pb.topk, nchunks, CT, scale_log2e, pb.qsh, pb.kvsh, pb.kvst, n_routed,
                          local_stride, share_window, ar);
  } else {
    hipLaunchKernelGGL((decode_split_kernel<T, D, U, AG>), dim3(grid), dim3(kDecodeThreads), 0, st,
                       static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V), idx,
                       part, pb.q_pos0, pb.Hq, pb.Hkv, S, AG ? S : pb.A, clip, pb.topk, nchunks, CT,
                       scale_log2e, pb.qsh, pb.kvsh, pb.kvst, n_routed, local_stride, share_window, ar);
  }
}

template <typename T, int D>
void launch_split(int grid, hipStream_t st, const void* Q, const void* K, const void* V,
                  const int32_t* idx, float* part, const Problem& pb, int S, int nchunks, int CT,
                  int n_routed, int local_stride, const AnchorRanges& ar) {
  const bool wide = wide_batches(CT);
  if (ar.on && wide)
    launch_split_u<T, D, 16, true>(grid, st, pb.prof_start, pb.prof_stop, Q, K, V, idx, part, pb, S, nchunks,
                                   CT, n_routed, local_stride, ar);
  else if (ar.on)
    launch_split_u<T, D, 8, true>(grid, st, pb.prof_start, pb.prof_stop, Q, K, V, idx, part, pb, S, nchunks,
                                  CT, n_routed, local_stride, ar);
  else if (wide)
    launch_split_u<T, D, 16, false>(grid, st, pb.prof_start, pb.prof_stop, Q, K, V, idx, part, pb, S, nchunks,
                                    CT, n_routed, local_stride, ar);
  else
    launch_split_u<T, D, 8, false>(grid, st, pb.prof_start, pb.prof_stop, Q, K, V, idx, part, pb, S, nchunks,
                                   CT, n_routed, local_stride, ar);
}

template <typename T, int D, int U, bool AG>
void launch_split_batched_u(int grid, int B, hipStream_t st, const sl_decode_seq* seqs, float* part,
                            int64_t part_stride, const Problem& pb, int S, int nchunks, int CT, int n_routed,
                            int local_stride, const AnchorBatch& ab) {
  const float scale_log2e = pb.scale * kLog2e;
  const int64_t kvsh = pb.kvsh_given ? pb.kvsh : (int64_t)0;
  const int A = AG ? S : pb.A;
  const bool clip = !AG && pb.A < pb.S && !pb.combined;
  const bool share_window = window_by_one_workgroup((int64_t)n_routed * B, CT, D, sizeof(T));
  hipLaunchKernelGGL((decode_split_batched_kernel<T, D, U, AG>), dim3(grid, B), dim3(kDecodeThreads), 0, st,
                     seqs, part, part_stride, pb.Hq, pb.Hkv, S, A, clip, pb.topk, nchunks, CT, scale_log2e,
                     pb.qsh, kvsh, pb.kvst, n_routed, local_stride, share_window, ab);
}

template <typename T, int D>
void launch_split_batched(int grid, int B, hipStream_t st, const sl_decode_seq* seqs, float* part,
                          int64_t part_stride, const Problem& pb, int S, int nchunks, int CT, int n_routed,
                          int local_stride, const AnchorBatch& ab) {
  const bool wide = wide_batches(CT);
  if (ab.on && wide)
    launch_split_batched_u<T, D, 16, true>(grid, B, st, seqs, part, part_stride, pb, S, nchunks, CT, n_routed,
                                           local_stride, ab);
  else if (ab.on)
    launch_split_batched_u<T, D, 8, true>(grid, B, st, seqs, part, part_stride, pb, S, nchunks, CT, n_routed,
                                          local_stride, ab);
  else if (wide)
    launch_split_batched_u<T, D, 16, false>(grid, B, st, seqs, part, part_stride, pb, S, nchunks, CT, n_routed,
                                            local_stride, ab);
  else
    launch_split_batched_u<T, D, 8, false>(grid, B, st, seqs, part, part_stride, pb, S, nchunks, CT, n_routed,
                                           local_stride, ab);
}

// The reductions keep one weight (joint form) or two statistics (gated form) per partial record of
// a head in dynamic LDS; a kernel gets 64 KB without asking for more.
inline bool reduce_fits_lds(int64_t nrec, bool combined) {
  return nrec * (combined ? 2 : 1) * (int64_t)sizeof(float) <= 64 * 1024;
}

int pick_chunk_tokens(const Problem& pb, int batch = 1) {
  // Aim for a few thousand workgroups so the 256 CUs keep enough loads in flight, without
  // going below 64 tokens per item.
  const int64_t units = (int64_t)batch * pb.Hq * (pb.topk + 1);
  int ct = 512;
  while (ct > 64 && units * ((pb.S + ct - 1) / ct) < 4096) ct >>= 1;
  return ct;
}

template <typename T, int D>
sl_status launch_decode(const Problem& pb, const void* Q, const void* K, const void* V,
                        const int32_t* idx, void* O, float* LSE, void* ws, hipStream_t st) {
  const int CT = pick_chunk_tokens(pb);
  const int nchunks = (pb.S + CT - 1) / CT;
  const int n_routed = pb.Hq * pb.topk * nchunks;
  const int local_stride = (int)align_up((size_t)pb.Hkv * nchunks, 8);
  const int grid = n_routed + pb.G * local_stride;
  float* part = static_cast<float*>(ws);
  const int nrec = (pb.topk + 1) * nchunks;
  if (!reduce_fits_lds(nrec, pb.combined)) return SL_ERR_UNSUPPORTED;  // before anything is enqueued
  launch_split<T, D>(grid, st, Q, K, V, idx, part, pb, pb.S, nchunks, CT, n_routed, local_stride,
                     AnchorRanges{false, 0, 0, 0, 0});
  if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
  if (pb.combined) {
    hipLaunchKernelGGL((decode_reduce_combined_kernel<T, D>), dim3(pb.Hq, D / kReduceDims), dim3(256),
                       (size_t)2 * nrec * sizeof(float), st, part, pb.gate, static_cast<T*>(O),
                       pb.topk, nchunks, nchunks);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
  }
  hipLaunchKernelGGL((decode_reduce_kernel<T, D>), dim3(pb.Hq, D / kReduceDims), dim3(256),
                     (size_t)nrec * sizeof(float), st, part, static_cast<T*>(O), LSE, nrec);
  if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
  return SL_OK;
}


// ------------------------------------------------------------------ the paper's own geometry
struct AnchorPlan {
  int64_t back, fwd, wlo, maxlen;
  int CT, nchunks, wchunks;
  size_t part_bytes, total_bytes;
};

AnchorPlan plan_anchor(const Problem& pb, int64_t window, int b, int f, int root, int batch = 1) {
  AnchorPlan a;
  const int64_t i = pb.q_pos0;
  const int64_t ell = span_base_length(i, root);  // l(i) = ceil(i^(1-p)), p = 1/root
  a.back = (int64_t)b * ell;
  a.fwd = (int64_t)f * ell;
  a.wlo = window > 0 ? (i - window + 1 > 0 ? i - window + 1 : 0) : i + 1;
  const int64_t wlen = i + 1 - a.wlo;
  a.maxlen = a.back + a.fwd + 1 > wlen ? a.back + a.fwd + 1 : wlen;
  if (a.maxlen > i + 1) a.maxlen = i + 1;
  const int64_t units = (int64_t)pb.Hq * (pb.topk + 1);
  int ct = 512;
  while (ct > 64 && batch * units * ((a.maxlen + ct - 1) / ct) < 4096) ct >>= 1;
  a.CT = ct;
  // chunks sit on the absolute CT-token lattice: a range of maxlen tokens touches one more of them
  // than its length alone fills
  a.nchunks = (int)((a.maxlen + ct - 1) / ct) + 1;
  a.wchunks = (int)((wlen + ct - 1) / ct) + 1;  // of the longest sequence; wlen <= maxlen
  if (a.wchunks > a.nchunks) a.wchunks = a.nchunks;
  a.part_bytes = align_up((size_t)batch * units * a.nchunks * (pb.D + 2) * sizeof(float), 256);
  a.total_bytes = a.part_bytes;
  return a;
}

template <typename T, int D>
sl_status launch_anchor_attention(const Problem& pb, const AnchorPlan& a, const void* Q,
                                  const void* K, const void* V, const int32_t* anchors, void* O,
                                  void* ws, hipStream_t st) {
  float* part = static_cast<float*>(ws);
  const AnchorRanges ar{true, a.wlo, a.back, a.fwd, a.wchunks};
  // every (head, slot, chunk) is a routed item here: the window is slot topk of every head, wchunks items
  const int grid = pb.Hq * (pb.topk * a.nchunks + a.wchunks);
  const int nrec = (pb.topk + 1) * a.nchunks;
  if (!reduce_fits_lds(nrec, true)) return SL_ERR_UNSUPPORTED;
  launch_split<T, D>(grid, st, Q, K, V, anchors, part, pb, 1, a.nchunks, a.CT, grid, 8, ar);
  if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
  hipLaunchKernelGGL((decode_reduce_combined_kernel<T, D>), dim3(pb.Hq, D / kReduceDims), dim3(256),
                     (size_t)2 * nrec * sizeof(float), st, part, pb.gate, static_cast<T*>(O), pb.topk,
                     a.nchunks, a.wchunks);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_decode_batched(const Problem& pb, const sl_decode_seq* seqs, int B, void* ws,
                                hipStream_t st) {
  const int CT = pick_chunk_tokens(pb, B);
  const int nchunks = (pb.S + CT - 1) / CT;
  const int nrec = (pb.topk + 1) * nchunks;
  if (!reduce_fits_lds(nrec, pb.combined)) return SL_ERR_UNSUPPORTED;
  const int64_t part_stride = (int64_t)pb.Hq * nrec * (D + 2);
  float* part = static_cast<float*>(ws);
  // same grid as the single-sequence launch in x, the sequence in y
  const int n_routed = pb.Hq * pb.topk * nchunks;
  const int local_stride = (int)align_up((size_t)pb.Hkv * nchunks, 8);
  const int grid = n_routed + pb.G * local_stride;
  launch_split_batched<T, D>(grid, B, st, seqs, part, part_stride, pb, pb.S, nchunks, CT, n_routed,
                             local_stride, AnchorBatch{false, 0, 0, 0, 2, 0});
  if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
  if (pb.combined)
    hipLaunchKernelGGL((decode_reduce_combined_batched_kernel<T, D>), dim3(pb.Hq, D / kReduceDims, B),
                       dim3(256), (size_t)2 * nrec * sizeof(float), st, seqs, part, part_stride, pb.topk,
                       nchunks, nchunks);
  else
    hipLaunchKernelGGL((decode_reduce_batched_kernel<T, D>), dim3(pb.Hq, D / kReduceDims, B), dim3(256),
                       (size_t)nrec * sizeof(float), st, seqs, part, part_stride, nrec);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_anchor_batched(const Problem& pb, const AnchorPlan& a, const AnchorBatch& ab,
                                const sl_decode_seq* seqs, int B, void* ws, hipStream_t st) {
  const int nrec = (pb.topk + 1) * a.nchunks;
  if (!reduce_fits_lds(nrec, true)) return SL_ERR_UNSUPPORTED;
  const int64_t part_stride = (int64_t)pb.Hq * nrec * (D + 2);
  float* part = static_cast<float*>(ws);
  const int grid = pb.Hq * (pb.topk * a.nchunks + a.wchunks);  // as for one sequence
  launch_split_batched<T, D>(grid, B, st, seqs, part, part_stride, pb, 1, a.nchunks, a.CT, grid, 8, ab);
  if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
  hipLaunchKernelGGL((decode_reduce_combined_batched_kernel<T, D>), dim3(pb.Hq, D / kReduceDims, B),
                     dim3(256), (size_t)2 * nrec * sizeof(float), st, seqs, part, part_stride, pb.topk,
                     a.nchunks, a.wchunks);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

}  // namespace

size_t decode_attention_batched_ws_bytes(const Problem& pb, int B) {
  const int CT = pick_chunk_tokens(pb, B);
  const int nchunks = (pb.S + CT - 1) / CT;
  return (size_t)B * pb.Hq * (pb.topk + 1) * nchunks * (pb.D + 2) * sizeof(float);
}

sl_status decode_attention_batched(const Problem& pb, const sl_decode_seq* seqs, int B, void* ws,
                                   hipStream_t st) {
  if (pb.dtype == SL_BF16) {
    if (pb.D == 128) return launch_decode_batched<bf16_t, 128>(pb, seqs, B, ws, st);
    return launch_decode_batched<bf16_t, 64>(pb, seqs, B, ws, st);
  }
  if (pb.D == 128) return launch_decode_batched<float, 128>(pb, seqs, B, ws, st);
  return launch_decode_batched<float, 64>(pb, seqs, B, ws, st);
}

size_t anchor_attention_batched_ws_bytes(const Problem& pb, int64_t window, int b, int f, int root,
                                         int B) {
  return plan_anchor(pb, window, b, f, root, B).total_bytes;
}

sl_status anchor_attention_decode_batched(const Problem& pb, int64_t window, int b, int f, int root,
                                          const sl_decode_seq* seqs, int B, void* ws, hipStream_t st) {
  const AnchorPlan a = plan_anchor(pb, window, b, f, root, B);
  const AnchorBatch ab{true, window, b, f, root, a.wchunks};
  if (pb.dtype == SL_BF16) {
    if (pb.D == 128) return launch_anchor_batched<bf16_t, 128>(pb, a, ab, seqs, B, ws, st);
    return launch_anchor_batched<bf16_t, 64>(pb, a, ab, seqs, B, ws, st);
  }
  if (pb.D == 128) return launch_anchor_batched<float, 128>(pb, a, ab, seqs, B, ws, st);
  return launch_anchor_batched<float, 64>(pb, a, ab, seqs, B, ws, st);
}

size_t decode_attention_ws_bytes(const Problem& pb) {
  const int CT = pick_chunk_tokens(pb);
  const int nchunks = (pb.S + CT - 1) / CT;
  return (size_t)pb.Hq * (pb.topk + 1) * nchunks * (pb.D + 2) * sizeof(float);
}

sl_status decode_attention(const Problem& pb, const void* Q, const void* K, const void* V,
                           const int32_t* idx, void* O, float* LSE, void* ws, hipStream_t st) {
  if (pb.dtype == SL_BF16) {
    if (pb.D == 128) return launch_decode<bf16_t, 128>(pb, Q, K, V, idx, O, LSE, ws, st);
    return launch_decode<bf16_t, 64>(pb, Q, K, V, idx, O, LSE, ws, st);
  }
  if (pb.D == 128) return launch_decode<float, 128>(pb, Q, K, V, idx, O, LSE, ws, st);
  return launch_decode<float, 64>(pb, Q, K, V, idx, O, LSE, ws, st);
}

}  // namespace sl

namespace sl {

size_t anchor_attention_ws_bytes(const Problem& pb, int64_t window, int b, int f, int root) {
  return plan_anchor(pb, window, b, f, root).total_bytes;
}

sl_status anchor_attention_decode(const Problem& pb, int64_t window, int b, int f, int root,
                                  const void* Q,
                                  const void* K, const void* V, const int32_t* anchors, void* O,
                                  void* ws, hipStream_t st) {
  const AnchorPlan a = plan_anchor(pb, window, b, f, root);
  if (pb.dtype == SL_BF16) {
    if (pb.D == 128) return launch_anchor_attention<bf16_t, 128>(pb, a, Q, K, V, anchors, O, ws, st);
    return launch_anchor_attention<bf16_t, 64>(pb, a, Q, K, V, anchors, O, ws, st);
  }
  if (pb.D == 128) return launch_anchor_attention<float, 128>(pb, a, Q, K, V, anchors, O, ws, st);
  return launch_anchor_attention<float, 64>(pb, a, Q, K, V, anchors, O, ws, st);
}

}  // namespace sl
