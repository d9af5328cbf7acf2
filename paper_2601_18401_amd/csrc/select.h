// Wavefront-level top-k selection over a score array held in LDS (eq. (3), TopK).
//
// k rounds of arg-max with removal.  Ties go to the lower span index: inside a lane candidates
// are visited in ascending index with a strict compare, and the cross-lane reduction prefers
// the lower index on equal scores.  The result is emitted in ascending index order, slots past
// min(k, c) are filled with -1 / -inf.
#pragma once

#include "sl_common.h"

namespace sl {

__device__ __forceinline__ void argmax_merge(float& v, int& j, float ov, int oj) {
  const bool take = (ov > v) || (ov == v && (unsigned)oj < (unsigned)j);
  v = take ? ov : v;
  j = take ? oj : j;
}

// sc: LDS array with the c candidate scores of one query row (private to this wavefront).
// All 64 lanes must call.  out_idx / out_scores point at the row's topk output slots.
__device__ __forceinline__ void wave_select_topk(float* sc, int c, int topk, int lane,
                                                 int32_t* __restrict__ out_idx,
                                                 float* __restrict__ out_scores) {
  const int kk = topk < c ? topk : c;
  int myj = 0x7fffffff;
  float mys = -INFINITY;
  for (int r = 0; r < kk; ++r) {
    float bv = -INFINITY;
    int bj = 0x7fffffff;
    for (int j = lane; j < c; j += 64) {
      const float v = sc[j];
      if (v > bv) {  // removed entries hold -inf and never win; scores are assumed finite
        bv = v;
        bj = j;
      }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const float ov = __shfl_xor(bv, off, 64);
      const int oj = __shfl_xor(bj, off, 64);
      argmax_merge(bv, bj, ov, oj);
    }
    if (lane == r) {
      myj = bj;
      mys = bv;
    }
    if (lane == 0 && bj != 0x7fffffff) sc[bj] = -INFINITY;  // remove the winner
    // LDS operations of one wavefront complete in issue order, so the next scan sees the removal;
    // the barrier only stops the compiler from moving code across it.
    __builtin_amdgcn_wave_barrier();
  }
  // ascending order: rank = number of selected indices below mine
  int rank = 0;
  for (int u = 0; u < kk; ++u) {
    const int ju = __shfl(myj, u, 64);
    rank += (ju < myj || (ju == myj && u < lane)) ? 1 : 0;  // second term only for non-finite input
  }
  if (lane < kk) {
    out_idx[rank] = myj == 0x7fffffff ? -1 : myj;
    if (out_scores) out_scores[rank] = mys;
  } else if (lane < topk) {
    out_idx[lane] = -1;
    if (out_scores) out_scores[lane] = -INFINITY;
  }
}

}  // namespace sl
