// Wavefront-level top-k selection over a score array held in LDS (eq. (3), TopK).
//
// k rounds of arg-max with removal.  The candidates are laid out lane-major: lane l owns the
// contiguous index range [l*R, (l+1)*R), so "lower lane" means "lower span index" and ties go
// to the lower index both inside a lane (ascending scan, strict compare) and across lanes
// (lowest lane among those holding the maximum).  The result is emitted in ascending index
// order; slots past min(k, c) are filled with -1 / -inf.
#pragma once

#include "sl_common.h"

namespace sl {

// Lane-major placement of c candidate scores in LDS: column of lane l starts at l * Rp floats.
// Rp is a multiple of 4 with Rp/4 odd, so 16-byte column reads of 16 consecutive lanes fall in
// distinct bank groups.
struct LaneMajor {
  int R, Rp;
  __host__ __device__ static LaneMajor make(int64_t c) {
    LaneMajor lm;
    lm.R = c > 0 ? (int)((c + 63) / 64) : 1;
    lm.Rp = (lm.R + 3) & ~3;
    if (((lm.Rp >> 2) & 1) == 0) lm.Rp += 4;
    return lm;
  }
  __host__ __device__ int lds_floats() const { return 64 * Rp; }
  __host__ __device__ int slot(int j) const { return (j / R) * Rp + (j % R); }
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float max_dpp_step(float v) {
  // lanes of rows outside ROW_MASK read back their own value (old = src): a harmless self-max
  const float ov = __int_as_float(
      __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
  return fmaxf(v, ov);
}

// Maximum over the 64 lanes without LDS traffic: butterfly inside each row of 16 lanes, then
// row broadcasts carry the row results up to lane 63, which is read back wave-uniform.
__device__ __forceinline__ float wave_max(float v) {
  v = max_dpp_step<0xB1, 0xF>(v);   // lane ^ 1
  v = max_dpp_step<0x4E, 0xF>(v);   // lane ^ 2
  v = max_dpp_step<0x141, 0xF>(v);  // other quad of the 8-lane half row
  v = max_dpp_step<0x140, 0xF>(v);  // other half of the 16-lane row
  v = max_dpp_step<0x142, 0xA>(v);  // rows 1, 3 <- last lane of rows 0, 2
  v = max_dpp_step<0x143, 0xC>(v);  // rows 2, 3 <- lane 31
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Every lane fills its own column with -inf (call before the scores are written).
__device__ __forceinline__ void select_clear(float* sc, const LaneMajor& lm, int lane) {
  float4* col = reinterpret_cast<float4*>(sc + lane * lm.Rp);
  const float4 ninf = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  for (int e4 = 0; e4 < lm.Rp / 4; ++e4) col[e4] = ninf;
}

// sc: lane-major LDS array with the c candidate scores of one query row (private to this
// wavefront), unused entries -inf.  Scores are assumed finite.  All 64 lanes must call.
// out_idx / out_scores point at the row's topk output slots.
// anchor_i >= 0: candidate j stands for the anchor token anchor_i - (anchor_s0 + j + 1)^root + 1
// of the stride pattern (Section 3.3, p = 1/root) and that token is what is written to out_idx.
__device__ __forceinline__ void wave_select_topk(float* sc, const LaneMajor& lm, int c, int topk,
                                                 int lane, int32_t* __restrict__ out_idx,
                                                 float* __restrict__ out_scores,
                                                 int64_t anchor_i = -1, int anchor_s0 = 0,
                                                 int anchor_root = 2) {
  const int kk = topk < c ? topk : c;
  float* colf = sc + lane * lm.Rp;
  const float4* col = reinterpret_cast<const float4*>(colf);
  const int n4 = lm.Rp / 4;
  int myj = 0x7fffffff;
  float mys = -INFINITY;
  for (int r = 0; r < kk; ++r) {
    float bv = -INFINITY;
    int be = 0;
    for (int e4 = 0; e4 < n4; e4 += 4) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = col[e4 + u < n4 ? e4 + u : n4 - 1];  // clamped re-reads never win
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = 4 * (e4 + u < n4 ? e4 + u : n4 - 1);
        if (v[u].x > bv) { bv = v[u].x; be = e; }
        if (v[u].y > bv) { bv = v[u].y; be = e + 1; }
        if (v[u].z > bv) { bv = v[u].z; be = e + 2; }
        if (v[u].w > bv) { bv = v[u].w; be = e + 3; }
      }
    }
    const float vmax = wave_max(bv);
    const unsigned long long holders = __ballot(bv == vmax && bv > -INFINITY);
    if (holders == 0ull) break;  // nothing finite left (only with non-finite input)
    const int wl = __ffsll((long long)holders) - 1;  // lowest lane = lowest span index
    const int wj = __builtin_amdgcn_readlane(lane * lm.R + be, wl);
    if (lane == wl) colf[be] = -INFINITY;  // remove the winner
    if (lane == r) {
      myj = wj;
      mys = vmax;
    }
    // LDS operations of one wavefront complete in issue order, so the next scan sees the
    // removal; the barrier only stops the compiler from moving code across it.
    __builtin_amdgcn_wave_barrier();
  }
  // ascending order: rank = number of selected indices below mine (empty picks sort last)
  int rank = 0;
  for (int u = 0; u < kk; ++u) {
    const int ju = __builtin_amdgcn_readlane(myj, u);
    rank += (ju < myj || (ju == myj && u < lane)) ? 1 : 0;
  }
  if (lane < kk) {
    if (anchor_i >= 0 && myj != 0x7fffffff) {
      // rank stays: ascending candidate = nearest anchor first
      myj = (int)anchor_token_of(anchor_i, (int64_t)anchor_s0 + myj, anchor_root);
    }
    out_idx[rank] = myj == 0x7fffffff ? -1 : myj;
    if (out_scores) out_scores[rank] = mys;
  } else if (lane < topk) {
    out_idx[lane] = -1;
    if (out_scores) out_scores[lane] = -INFINITY;
  }
}


// Inclusive prefix sum over the 64 lanes (DPP only): Hillis-Steele inside each row of 16 lanes
// (row_shr 1, 2, 4, 8 with zero fill), then the row totals ripple up through row broadcasts.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int scan_dpp_step(int v) {
  return v + __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, true);
}
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v = scan_dpp_step<0x111, 0xF>(v);
  v = scan_dpp_step<0x112, 0xF>(v);
  v = scan_dpp_step<0x114, 0xF>(v);
  v = scan_dpp_step<0x118, 0xF>(v);
  v = scan_dpp_step<0x142, 0xA>(v);  // rows 1, 3 += total of rows 0, 2
  v = scan_dpp_step<0x143, 0xC>(v);  // rows 2, 3 += total of rows 0..1
  return v;
}

}  // namespace sl
