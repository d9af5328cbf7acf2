// Row-stationary prefill span-attention: one wavefront per (head, query row) streams the rows
// of the selected spans and of the local window (eq. (4) over the de-duplicated union,
// Algorithm 1) with an online softmax.  Exact and simple; used for fp32 and for shapes the
// matrix-core path does not cover.
#include "kernels.h"
#include "stream_attend.h"

namespace sl {

namespace {

// Merges the row groups of a wavefront (lanes with equal lane % LPR hold the same d-slice); on
// return every lane holds the state of all rows the wavefront attended.
template <typename T, int D>
__device__ __forceinline__ void merge_row_groups(AttendState<T, D>& st) {
  constexpr int EPL = RowLayout<T, D>::EPL, LPR = RowLayout<T, D>::LPR;
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
    const float mo = __shfl_xor(st.m, off, 64);
    const float lo = __shfl_xor(st.l, off, 64);
    const float M = fmaxf(st.m, mo);
    const float wa = st.m > -INFINITY ? fast_exp2(st.m - M) : 0.f;
    const float wb = mo > -INFINITY ? fast_exp2(mo - M) : 0.f;
    st.l = st.l * wa + lo * wb;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float oo = __shfl_xor(st.o[e], off, 64);
      st.o[e] = st.o[e] * wa + oo * wb;
    }
    st.m = M;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_attention_rows_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ idx, T* __restrict__ O, float* __restrict__ LSE, int64_t Lq,
    int64_t q_pos0, int Hq, int G, int S, int A, int topk, float scale_log2e, int64_t qsh, int64_t qst,
    int64_t kvsh, int64_t kvst) {
  // Anchors every A tokens, span j = the S tokens ending at (j+1)*A - 1 (A = S: the disjoint grid).
  // With A < S the spans of a row overlap: a span's range then starts behind the end of the
  // nearest lower span the row lists, so that every token of the union is attended once.
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + wave;
  if (row >= (int64_t)Hq * Lq) return;
  const int h = (int)(row / Lq);
  const int64_t r = row % Lq, i = q_pos0 + r;
  const int kv = h / G;
  const int64_t c = i / A;
  const int lr = lane % LPR;
  float q2[EPL];
  {
    float qf[EPL];
    Elem<T>::unpack(load16(Q + h * qsh + r * qst + lr * EPL), qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) q2[e] = qf[e] * scale_log2e;
  }
  const T* Kb = K + kv * kvsh;
  const T* Vb = V + kv * kvsh;
  AttendState<T, D> st;
  st.init();
  for (int slot = 0; slot < topk; ++slot) {
    const int64_t j = idx[row * topk + slot];
    if (j >= 0 && j < c) {
      const int64_t end = (j + 1) * A;
      int64_t begin = end - S > 0 ? end - S : 0;
      if (A < S) {
        for (int s2 = 0; s2 < topk; ++s2) {
          const int64_t jj = idx[row * topk + s2];
          if (jj >= 0 && jj < j && (jj + 1) * A > begin) begin = (jj + 1) * A;
        }
      }
      attend_range<T, D, 4>(q2, Kb, Vb, kvst, begin, end, lane, st);
    }
  }
  attend_range<T, D, 4>(q2, Kb, Vb, kvst, c * A, i + 1, lane, st);

  merge_row_groups<T, D>(st);
  if (lane < LPR) {
    const float inv = 1.f / st.l;  // the local window always holds the query's own token: l > 0
    T* op = O + row * D + lr * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) Elem<T>::store1(op + e, st.o[e] * inv);
    if (lane == 0) LSE[row] = (st.m + __log2f(st.l)) * kLn2;
  }
}


// Combination form (Section 3.4, eq. (5)-(6); Algorithm 1): per valid slot t the attention A_t
// over span t and the local window with its own softmax, O = sum_t alpha_t A_t with
// alpha = softmax of the slots' search scores; no valid slot: the window alone.  The window is
// streamed once and its (m, l, o) state is merged into every span's state.
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_combined_rows_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ idx, const float* __restrict__ gate, T* __restrict__ O, int64_t Lq,
    int64_t q_pos0, int Hq, int G, int S, int A, int topk, float scale_log2e, int64_t qsh, int64_t qst,
    int64_t kvsh, int64_t kvst) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + wave;
  if (row >= (int64_t)Hq * Lq) return;
  const int h = (int)(row / Lq);
  const int64_t r = row % Lq, i = q_pos0 + r;
  const int kv = h / G;
  const int64_t c = i / A;  // anchors every A tokens; every span has its own softmax: no clipping here
  const int lr = lane % LPR;
  float q2[EPL];
  {
    float qf[EPL];
    Elem<T>::unpack(load16(Q + h * qsh + r * qst + lr * EPL), qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) q2[e] = qf[e] * scale_log2e;
  }
  const T* Kb = K + kv * kvsh;
  const T* Vb = V + kv * kvsh;
  AttendState<T, D> win;
  win.init();
  attend_range<T, D, 4>(q2, Kb, Vb, kvst, c * A, i + 1, lane, win);
  merge_row_groups<T, D>(win);  // the window always holds the query's own token: win.l > 0

  // gate: softmax of the scores of the valid slots
  float smax = -INFINITY;
  for (int slot = 0; slot < topk; ++slot) {
    const int64_t j = idx[row * topk + slot];
    if (j >= 0 && j < c) smax = fmaxf(smax, gate[row * topk + slot]);
  }
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  float asum = 0.f;
  for (int slot = 0; slot < topk; ++slot) {
    const int64_t j = idx[row * topk + slot];
    if (!(j >= 0 && j < c)) continue;
    AttendState<T, D> st;
    st.init();
    attend_range<T, D, 4>(q2, Kb, Vb, kvst, (j + 1) * A - S > 0 ? (j + 1) * A - S : 0, (j + 1) * A, lane, st);
    merge_row_groups<T, D>(st);
    const float M = fmaxf(st.m, win.m);
    const float wa = fast_exp2(st.m - M), wb = fast_exp2(win.m - M);
    const float a = __expf(gate[row * topk + slot] - smax);
    const float f = a / (st.l * wa + win.l * wb);
    asum += a;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = fmaf(f, st.o[e] * wa + win.o[e] * wb, acc[e]);
  }
  if (lane < LPR) {
    T* op = O + row * D + lr * EPL;
    const bool any = asum > 0.f;
    const float inv = any ? 1.f / asum : 1.f / win.l;
#pragma unroll
    for (int e = 0; e < EPL; ++e) Elem<T>::store1(op + e, (any ? acc[e] : win.o[e]) * inv);
  }
}

// The paper's geometry, prefill form, attention + combination (Section 3.3-3.4, Algorithm 1):
// for the query at position i, l = ceil(i^(1-p)) with p = 1/root, W = [max(0, i - window + 1), i], and per
// selected anchor t the span S_t = [max(0, t - b*l), min(i, t + f*l)].  DedupConcat(S_t, W) is S_t
// clipped at the start of W followed by W (W is a suffix of [0, i]); A_t has its own softmax and
// O = sum_t alpha_t A_t with alpha = softmax of the slots' search scores; no valid slot: W alone
// (zeros if there is no window either).  The window is streamed once per row.
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_anchor_combined_rows_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ anchors, const float* __restrict__ gate, T* __restrict__ O,
    int64_t Lq, int64_t q_pos0, int Hq, int G, int topk, int64_t window, int b, int f, int root,
    float scale_log2e, int64_t qsh, int64_t qst, int64_t kvsh, int64_t kvst) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * 4 + wave;
  if (row >= (int64_t)Hq * Lq) return;
  const int h = (int)(row / Lq);
  const int64_t r = row % Lq, i = q_pos0 + r;
  const int kv = h / G;
  const int64_t ell = span_base_length(i, root);
  const int64_t back = b * ell, fwd = f * ell;
  const int64_t wlo = window > 0 ? (i - window + 1 > 0 ? i - window + 1 : 0) : i + 1;
  const int lr = lane % LPR;
  float q2[EPL];
  {
    float qf[EPL];
    Elem<T>::unpack(load16(Q + h * qsh + r * qst + lr * EPL), qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) q2[e] = qf[e] * scale_log2e;
  }
  const T* Kb = K + kv * kvsh;
  const T* Vb = V + kv * kvsh;
  AttendState<T, D> win;
  win.init();
  attend_range<T, D, 4>(q2, Kb, Vb, kvst, wlo, i + 1, lane, win);
  merge_row_groups<T, D>(win);  // empty window: win.m = -inf, win.l = 0

  float smax = -INFINITY;
  for (int slot = 0; slot < topk; ++slot) {
    const int64_t t = anchors[row * topk + slot];
    if (t >= 0 && t <= i) smax = fmaxf(smax, gate[row * topk + slot]);
  }
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  float asum = 0.f;
  for (int slot = 0; slot < topk; ++slot) {
    const int64_t t = anchors[row * topk + slot];
    if (!(t >= 0 && t <= i)) continue;
    const int64_t r0 = t - back > 0 ? t - back : 0;
    const int64_t e1 = t + fwd < i ? t + fwd : i;
    int64_t r1 = (e1 < wlo - 1 ? e1 : wlo - 1) + 1;
    r1 = r1 < r0 ? r0 : r1;
    AttendState<T, D> st;
    st.init();
    attend_range<T, D, 4>(q2, Kb, Vb, kvst, r0, r1, lane, st);
    merge_row_groups<T, D>(st);
    const float M = fmaxf(st.m, win.m);
    const float wa = st.m > -INFINITY ? fast_exp2(st.m - M) : 0.f;
    const float wb = win.m > -INFINITY ? fast_exp2(win.m - M) : 0.f;
    const float den = st.l * wa + win.l * wb;
    const float a = __expf(gate[row * topk + slot] - smax);
    const float fct = den > 0.f ? a / den : 0.f;
    asum += a;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = fmaf(fct, st.o[e] * wa + win.o[e] * wb, acc[e]);
  }
  if (lane < LPR) {
    T* op = O + row * D + lr * EPL;
    const bool any = asum > 0.f;
    const float inv = any ? 1.f / asum : (win.l > 0.f ? 1.f / win.l : 0.f);
#pragma unroll
    for (int e = 0; e < EPL; ++e) Elem<T>::store1(op + e, (any ? acc[e] : win.o[e]) * inv);
  }
}

template <typename T, int D>
sl_status launch_anchor_rows(const Problem& pb, int64_t window, int b, int f, int root, const void* Q,
                             const void* K, const void* V, const int32_t* anchors, void* O,
                             hipStream_t st) {
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  hipLaunchKernelGGL((prefill_anchor_combined_rows_kernel<T, D>), dim3((unsigned)((rows + 3) / 4)),
                     dim3(256), 0, st, static_cast<const T*>(Q), static_cast<const T*>(K),
                     static_cast<const T*>(V), anchors, pb.gate, static_cast<T*>(O), pb.Lq, pb.q_pos0,
                     pb.Hq, pb.G, pb.topk, window, b, f, root, pb.scale * kLog2e, pb.qsh, pb.qst, pb.kvsh,
                     pb.kvst);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_rows(const Problem& pb, const void* Q, const void* K, const void* V,
                      const int32_t* idx, void* O, float* LSE, hipStream_t st) {
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  if (pb.combined) {
    hipLaunchKernelGGL((prefill_combined_rows_kernel<T, D>), dim3((unsigned)((rows + 3) / 4)),
                       dim3(256), 0, st, static_cast<const T*>(Q), static_cast<const T*>(K),
                       static_cast<const T*>(V), idx, pb.gate, static_cast<T*>(O), pb.Lq, pb.q_pos0,
                       pb.Hq, pb.G, pb.S, pb.A, pb.topk, pb.scale * kLog2e, pb.qsh, pb.qst, pb.kvsh,
                       pb.kvst);
    if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
  }
  hipLaunchKernelGGL((prefill_attention_rows_kernel<T, D>), dim3((unsigned)((rows + 3) / 4)),
                     dim3(256), 0, st, static_cast<const T*>(Q), static_cast<const T*>(K),
                     static_cast<const T*>(V), idx, static_cast<T*>(O), LSE, pb.Lq, pb.q_pos0,
                     pb.Hq, pb.G, pb.S, pb.A, pb.topk, pb.scale * kLog2e, pb.qsh, pb.qst, pb.kvsh,
                     pb.kvst);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

}  // namespace

sl_status prefill_attention_rows(const Problem& pb, const void* Q, const void* K, const void* V,
                                 const int32_t* idx, void* O, float* LSE, hipStream_t st) {
  if (pb.dtype == SL_BF16) {
    if (pb.D == 128) return launch_rows<bf16_t, 128>(pb, Q, K, V, idx, O, LSE, st);
    return launch_rows<bf16_t, 64>(pb, Q, K, V, idx, O, LSE, st);
  }
  if (pb.D == 128) return launch_rows<float, 128>(pb, Q, K, V, idx, O, LSE, st);
  return launch_rows<float, 64>(pb, Q, K, V, idx, O, LSE, st);
}

sl_status anchor_attention_prefill(const Problem& pb, int64_t window, int b, int f, int root,
                                   const void* Q,
                                   const void* K, const void* V, const int32_t* anchors, void* O,
                                   hipStream_t st) {
  if (pb.dtype == SL_BF16) {
    if (pb.D == 128) return launch_anchor_rows<bf16_t, 128>(pb, window, b, f, root, Q, K, V, anchors, O, st);
    return launch_anchor_rows<bf16_t, 64>(pb, window, b, f, root, Q, K, V, anchors, O, st);
  }
  if (pb.D == 128) return launch_anchor_rows<float, 128>(pb, window, b, f, root, Q, K, V, anchors, O, st);
  return launch_anchor_rows<float, 64>(pb, window, b, f, root, Q, K, V, anchors, O, st);
}

}  // namespace sl
