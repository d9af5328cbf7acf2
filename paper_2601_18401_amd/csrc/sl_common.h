// Shared host/device helpers for the gfx950 kernels of the span-search / span-attention library.
#pragma once

#include <cmath>

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sl.h"

namespace sl {

// Host-side, validated view of sl_params with defaults resolved.
struct Problem {
  int64_t L, Lq, q_pos0;
  int Hq, Hkv, G, D, S, topk;
  int A;  // anchor spacing (sl_params.span_stride, S if not given): c = i / A, span j = [max(0, (j+1)A - S), (j+1)A)
  int dtype;
  float scale;  // resolved softmax scale
  int64_t qsh, qst, kvsh, kvst;
  bool kvsh_given;  // the caller gave a kv head stride (else kvsh = L * kvst: packed)
  int64_t n;  // ceil(L / A): rows of the span-key tensor, spans of the grid
  hipEvent_t prof_start, prof_stop;
  // Combination (Section 3.4) instead of one joint softmax over the selected spans and the
  // window; gate = search scores [Hq][Lq][topk] of the slots of idx (unread when topk == 0).
  bool combined;
  const float* gate;
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- device helpers
#if defined(__HIPCC__)

typedef uint16_t bf16_t;  // raw bfloat16 storage

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int EPL = 4;  // elements per 16-byte lane load
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x);
    f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z);
    f[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ float load1(const float* p) { return *p; }
  __device__ static __forceinline__ void store1(float* p, float v) { *p = v; }
};
template <>
struct Elem<bf16_t> {
  static constexpr int EPL = 8;
  __device__ static __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x << 16);
    f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16);
    f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16);
    f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16);
    f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float load1(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store1(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Dot product of two 16-byte row pieces on top of acc, as every span-search kernel takes it
// (eq. (2)): the same instructions in the same order everywhere, so that the kernels agree bit for
// bit.  bf16: four two-element dot instructions on the packed pairs (exact products, fp32 sums) -
// no unpacking; fp32: a chain of four fused multiply-adds.
template <typename T>
struct Piece;
template <>
struct Piece<float> {
  __device__ static __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
    acc = fmaf(__uint_as_float(a.x), __uint_as_float(b.x), acc);
    acc = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), acc);
    acc = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), acc);
    acc = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), acc);
    return acc;
  }
};
template <>
struct Piece<bf16_t> {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  __device__ static __forceinline__ float dot2(unsigned a, unsigned b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
  }
  __device__ static __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
    acc = dot2(a.x, b.x, acc);
    acc = dot2(a.y, b.y, acc);
    acc = dot2(a.z, b.z, acc);
    acc = dot2(a.w, b.w, acc);
    return acc;
  }
};

// One row of D elements is covered by LPR lanes, each holding 16 bytes; a wavefront of 64
// lanes covers RPW rows per load instruction.
template <typename T, int D>
struct RowLayout {
  static constexpr int EPL = Elem<T>::EPL;
  static constexpr int LPR = D / EPL;
  static constexpr int RPW = 64 / LPR;
  static_assert(LPR >= 8 && LPR <= 32, "unsupported row width");
};

__device__ __forceinline__ uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// 16-byte load with the non-temporal hint, for data that is read once
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte store with the non-temporal hint, for data that is not read again soon
__device__ __forceinline__ void store16_stream(void* p, uint4 v) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
}

// ---- the paper's anchor geometry (Section 3.3) for p = 1/root, root = 2 or 3, in exact integer
// arithmetic.  Valid for 0 <= x < 2^62.
__host__ __device__ inline int64_t ipow_root(int64_t v, int root) { return root == 2 ? v * v : v * v * v; }
// floor(x^(1/root))
__host__ __device__ inline int64_t iroot_floor(int64_t x, int root) {
  if (x <= 0) return 0;
  int64_t m = (int64_t)(root == 2 ? sqrt((double)x) : cbrt((double)x));
  while (m > 0 && ipow_root(m, root) > x) --m;
  while (ipow_root(m + 1, root) <= x) ++m;
  return m;
}
// anchor token of stride index s for the query at position i: i - (s+1)^root + 1
__host__ __device__ inline int64_t anchor_token_of(int64_t i, int64_t s, int root) {
  return i - ipow_root(s + 1, root) + 1;
}
// l(i) = ceil(i^(1-p)) = the smallest m with m^root >= i^(root-1); i < 2^31
__host__ __device__ inline int64_t span_base_length(int64_t i, int root) {
  if (i <= 0) return 0;
  const int64_t target = root == 2 ? i : i * i;
  const int64_t m = iroot_floor(target, root);
  return ipow_root(m, root) == target ? m : m + 1;
}

// DPP lane exchange (no LDS traffic). ctrl: quad_perm 0x00-0xFF, row_shl:n 0x100+n, row_shr:n 0x110+n,
// row_ror:n 0x120+n, row_mirror 0x140, row_half_mirror 0x141.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over the LPR consecutive lanes of a row group; every lane of the group gets the total.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_f32<0xB1>(v);   // lane ^ 1
  v += dpp_f32<0x4E>(v);   // lane ^ 2
  v += dpp_f32<0x141>(v);  // mirror within 8 lanes: adds the other quad
  if (LPR >= 16) v += dpp_f32<0x140>(v);  // mirror within 16 lanes: adds the other half-row
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

// Eight values per lane (a[0..7]) summed over the LPR lanes of a row group, each lane ending up
// with the total of ONE of them: lane lr gets the group sum of a[lr % 8].  A reduce-scatter: at
// every level a lane passes on the half of its values that its partner keeps and adds what it
// receives to the half it keeps (24 instructions for 16 lanes, where eight group_sum calls take 32
// and the caller a select per value on top).  The additions pair the same partial sums as
// group_sum does, level by level, so the totals are bit-identical to it.
template <int LPR>
__device__ __forceinline__ float group_sum_scatter8(const float (&a)[8], int lr) {
  static_assert(LPR >= 8, "needs a lane per value");
  const bool b0 = lr & 1, b1 = lr & 2, b2 = lr & 4;
  float l1[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {  // l1[j]: the pair's sum of value 2j + b0
    const float keep = b0 ? a[2 * j + 1] : a[2 * j], send = b0 ? a[2 * j] : a[2 * j + 1];
    l1[j] = keep + dpp_f32<0xB1>(send);   // lane ^ 1
  }
  float l2[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {  // l2[j]: the quad's sum of value 4j + 2*b1 + b0
    const float keep = b1 ? l1[2 * j + 1] : l1[2 * j], send = b1 ? l1[2 * j] : l1[2 * j + 1];
    l2[j] = keep + dpp_f32<0x4E>(send);   // lane ^ 2
  }
  const float keep = b2 ? l2[1] : l2[0], send = b2 ? l2[0] : l2[1];
  // lane ^ 4: rows shifted by four lanes either way, each written to the banks it is right for
  int other = __builtin_amdgcn_update_dpp(0, __float_as_int(send), 0x104, 0xF, 0x5, false);      // row_shl:4 -> lanes 0-3, 8-11
  other = __builtin_amdgcn_update_dpp(other, __float_as_int(send), 0x114, 0xF, 0xA, false);      // row_shr:4 -> lanes 4-7, 12-15
  float v = keep + __int_as_float(other);  // value 4*b2 + 2*b1 + b0 = lr % 8, summed over 8 lanes
  if (LPR >= 16) v += dpp_f32<0x128>(v);   // row rotated by 8 = lane ^ 8: the other half-row's sum of the same value
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

#endif  // __HIPCC__

}  // namespace sl
