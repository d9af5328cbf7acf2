// Wavefront-level streaming attention over a contiguous token range, one query vector.
//
// Used where the work is a matrix-vector product per query (decode, and the row-stationary
// prefill path): the K/V rows are read exactly once with 16-byte-per-lane coalesced loads,
// LPR lanes cover one row and a wavefront covers RPW rows per load instruction.  Each row group
// keeps its own online-softmax state (m, l, o), in log2 units; groups are merged by the caller.
#pragma once

#include "sl_common.h"

namespace sl {

template <typename T, int D>
struct AttendState {
  static constexpr int EPL = RowLayout<T, D>::EPL;
  float m;       // running max of logit * log2(e)
  float l;       // running sum of 2^(z - m)
  float o[EPL];  // running sum of 2^(z - m) * V[:, d-slice of this lane]
  __device__ __forceinline__ void init() {
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;
  }
};

// q2[e]: this lane's slice of the query, already multiplied by scale * log2(e).
// Kb/Vb: base of the kv head; row t starts at Kb + t * stride_t (elements).
// Tokens [t0, t1) are attended; t0 < t1 is not required (empty range is a no-op).
// STREAM: the rows are loaded with the non-temporal hint (read once, no reuse expected from the
// caches); a read-only stream sustains about 12 % more HBM bandwidth that way on this part.
// One batch of the stream: U K loads and U V loads per lane, rows tb + u * RPW + g, clamped into
// [.., t1) (rows past the end are loaded from the last row and masked by attend_loaded).
template <typename T, int D, int U, bool STREAM>
__device__ __forceinline__ void load_rows(const T* __restrict__ Kb, const T* __restrict__ Vb, int64_t stride_t,
                                          int64_t tb, int64_t t1, int lane, uint4 (&kr)[U], uint4 (&vr)[U]) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  const int g = lane / LPR, lr = lane % LPR;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t tok = tb + u * RPW + g;
    tok = tok < t1 ? tok : t1 - 1;  // clamp: stays inside the range, masked below
    kr[u] = STREAM ? load16_stream(Kb + tok * stride_t + lr * EPL) : load16(Kb + tok * stride_t + lr * EPL);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t tok = tb + u * RPW + g;
    tok = tok < t1 ? tok : t1 - 1;
    vr[u] = STREAM ? load16_stream(Vb + tok * stride_t + lr * EPL) : load16(Vb + tok * stride_t + lr * EPL);
  }
}

// Online-softmax update of st with the batch that load_rows fetched for rows tb, tb + 1, ...:
// the rows inside [lo, hi) are attended, the others masked.
// (I: int64_t token positions, or int offsets from a common base.)
template <typename T, int D, int U, typename I>
__device__ __forceinline__ void attend_loaded(const float* q2, const uint4 (&kr)[U], const uint4 (&vr)[U],
                                              I tb, I lo, I hi, int lane, AttendState<T, D>& st) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  const int g = lane / LPR;
  float s[U];
  float bm = -INFINITY;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float kf[EPL];
    Elem<T>::unpack(kr[u], kf);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc = fmaf(q2[e], kf[e], acc);
    acc = group_sum<LPR>(acc);
    const I tok = tb + u * RPW + g;
    s[u] = (tok >= lo && tok < hi) ? acc : -INFINITY;
    bm = fmaxf(bm, s[u]);
  }
  const float m_new = fmaxf(st.m, bm);
  if (m_new > -INFINITY) {
    const float corr = fast_exp2(st.m - m_new);  // st.m = -inf -> 0
    st.l *= corr;
#pragma unroll
    for (int e = 0; e < EPL; ++e) st.o[e] *= corr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float p = fast_exp2(s[u] - m_new);
      st.l += p;
      float vf[EPL];
      Elem<T>::unpack(vr[u], vf);
#pragma unroll
      for (int e = 0; e < EPL; ++e) st.o[e] = fmaf(p, vf[e], st.o[e]);
    }
    st.m = m_new;
  }
}

template <typename T, int D, int U, bool STREAM = false>
__device__ __forceinline__ void attend_range(const float* q2, const T* __restrict__ Kb,
                                             const T* __restrict__ Vb, int64_t stride_t, int64_t t0,
                                             int64_t t1, int lane, AttendState<T, D>& st) {
  constexpr int RPW = RowLayout<T, D>::RPW;
  for (int64_t tb = t0; tb < t1; tb += RPW * U) {
    uint4 kr[U], vr[U];
    load_rows<T, D, U, STREAM>(Kb, Vb, stride_t, tb, t1, lane, kr, vr);
    attend_loaded<T, D, U>(q2, kr, vr, tb, t0, t1, lane, st);
  }
}

}  // namespace sl
