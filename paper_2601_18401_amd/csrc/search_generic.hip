// Span-search kernels that need no matrix cores: the span-key gather, the decode form
// (one workgroup per head scores its candidates into LDS and selects) and the
// row-stationary prefill form (one wavefront per query row) used for fp32 and for shapes the
// MFMA path does not cover.
//
// Scores are eq. (2): raw dot products, accumulated in fp32 from exact products.
#include "kernels.h"
#include "select.h"

namespace sl {

namespace {

// ------------------------------------------------------------------ a0: span keys
template <typename T, int D>
__global__ __launch_bounds__(256) void span_keys_kernel(const T* __restrict__ K, T* __restrict__ Ks,
                                                        int64_t nfull, int64_t n, int S,
                                                        int64_t kvsh, int64_t kvst) {
  using RL = RowLayout<T, D>;
  const int64_t row = (int64_t)blockIdx.x * (256 / RL::LPR) + threadIdx.x / RL::LPR;
  const int lr = threadIdx.x % RL::LPR;
  const int kv = blockIdx.y;
  if (row >= nfull) return;
  const uint4 v = load16(K + kv * kvsh + ((row + 1) * S - 1) * kvst + lr * RL::EPL);
  *reinterpret_cast<uint4*>(Ks + ((int64_t)kv * n + row) * D + lr * RL::EPL) = v;
}

// Address of the search key of span j for kv head `kv`: packed Ks row, or K at the anchor.
template <typename T, int D>
__device__ __forceinline__ const T* span_key_ptr(const T* K, const T* Ks, int kv, int64_t j,
                                                 int64_t n, int S, int64_t kvsh, int64_t kvst) {
  return Ks ? Ks + ((int64_t)kv * n + j) * D : K + kv * kvsh + ((j + 1) * S - 1) * kvst;
}

// ------------------------------------------------------------------ a7: decode search
// One workgroup of 16 wavefronts per query head: the wavefronts score the head's c candidate
// span keys into LDS (RPW keys per load instruction, 16-byte lanes), then wavefront 0 selects.
// Heads of one kv group re-read the same keys; they are a few hundred KB and L2-resident.
constexpr int kDecodeSearchThreads = 1024;

template <typename T, int D>
__global__ __launch_bounds__(kDecodeSearchThreads) void decode_search_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, const T* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t c, int64_t n, int G, int S,
    int topk, int64_t qsh, int64_t kvsh, int64_t kvst) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  // 16 independent 16-byte loads per lane are in flight before the first use: a head's whole
  // candidate set is covered in one to three memory round trips
  constexpr int U = 16, NW = kDecodeSearchThreads / 64;
  extern __shared__ float s_sc[];  // lane-major score array of the selecting wavefront
  const int h = blockIdx.x, kv = h / G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane / LPR, lr = lane % LPR;
  const LaneMajor lm = LaneMajor::make(c);
  if (wave == 0) select_clear(s_sc, lm, lane);
  float qf[EPL];
  Elem<T>::unpack(load16(Qs + (int64_t)h * qsh + lr * EPL), qf);
  __syncthreads();
  for (int64_t jb = (int64_t)wave * RPW * U; jb < c; jb += NW * RPW * U) {
    uint4 kr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t j = jb + u * RPW + g;
      j = j < c ? j : c - 1;
      kr[u] = load16(span_key_ptr<T, D>(K, Ks, kv, j, n, S, kvsh, kvst) + lr * EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      Elem<T>::unpack(kr[u], kf);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc = fmaf(qf[e], kf[e], acc);
      acc = group_sum<LPR>(acc);
      const int64_t j = jb + u * RPW + g;
      if (lr == 0 && j < c) s_sc[lm.slot((int)j)] = acc;
    }
  }
  __syncthreads();
  if (wave == 0)
    wave_select_topk(s_sc, lm, (int)c, topk, lane, idx + (int64_t)h * topk,
                     scores ? scores + (int64_t)h * topk : nullptr);
}

// ------------------------------------------------------------------ a1 + a2: prefill, row-stationary
// One wavefront per (head, query row); W rows per workgroup; dynamic LDS = W lane-major score arrays.
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_search_rows_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, const T* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t Lq, int64_t q_pos0, int Hq,
    int G, int S, int topk, int64_t n, int W, int lds_per_wave, int64_t qsh, int64_t qst,
    int64_t kvsh, int64_t kvst) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  extern __shared__ float s_all[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * W + wave;
  if (wave >= W || row >= (int64_t)Hq * Lq) return;
  float* sc = s_all + (int64_t)wave * lds_per_wave;
  const int h = (int)(row / Lq);
  const int64_t r = row % Lq, i = q_pos0 + r;
  const int kv = h / G;
  const int64_t c = i / S;
  const int g = lane / LPR, lr = lane % LPR;
  const LaneMajor lm = LaneMajor::make(c);
  select_clear(sc, lm, lane);
  __builtin_amdgcn_wave_barrier();
  float qf[EPL];
  Elem<T>::unpack(load16(Qs + h * qsh + r * qst + lr * EPL), qf);
  constexpr int U = 4;
  for (int64_t jb = 0; jb < c; jb += RPW * U) {
    uint4 kr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t j = jb + u * RPW + g;
      j = j < c ? j : c - 1;
      kr[u] = load16(span_key_ptr<T, D>(K, Ks, kv, j, n, S, kvsh, kvst) + lr * EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPL];
      Elem<T>::unpack(kr[u], kf);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc = fmaf(qf[e], kf[e], acc);
      acc = group_sum<LPR>(acc);
      const int64_t j = jb + u * RPW + g;
      if (lr == 0 && j < c) sc[lm.slot((int)j)] = acc;
    }
  }
  __builtin_amdgcn_wave_barrier();
  wave_select_topk(sc, lm, (int)c, topk, lane, idx + row * topk,
                   scores ? scores + row * topk : nullptr);
}

template <typename T, int D>
sl_status launch_span_keys(const Problem& pb, const void* K, void* Ks, hipStream_t st) {
  using RL = RowLayout<T, D>;
  const int64_t nfull = pb.L / pb.S;
  if (nfull == 0) return SL_OK;
  const int rows_per_block = 256 / RL::LPR;
  dim3 grid((unsigned)((nfull + rows_per_block - 1) / rows_per_block), pb.Hkv);
  hipLaunchKernelGGL((span_keys_kernel<T, D>), grid, dim3(256), 0, st, static_cast<const T*>(K),
                     static_cast<T*>(Ks), nfull, pb.n, pb.S, pb.kvsh, pb.kvst);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_decode_search(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                               int32_t* idx, float* scores, hipStream_t st) {
  const int64_t c = pb.q_pos0 / pb.S;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  hipLaunchKernelGGL((decode_search_kernel<T, D>), dim3(pb.Hq), dim3(kDecodeSearchThreads),
                     (size_t)LaneMajor::make(c).lds_floats() * sizeof(float), st,
                     static_cast<const T*>(Qs),
                     static_cast<const T*>(K), static_cast<const T*>(Ks), idx, scores, c, pb.n,
                     pb.G, pb.S, pb.topk, pb.qsh, pb.kvsh, pb.kvst);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_prefill_search_rows(const Problem& pb, const void* Qs, const void* K,
                                     const void* Ks, int32_t* idx, float* scores,
                                     hipStream_t st) {
  // the widest row (last query) sizes the per-wavefront score array
  const int lds_per_wave = LaneMajor::make((pb.q_pos0 + pb.Lq - 1) / pb.S).lds_floats();
  int W = 4;
  while (W > 1 && (size_t)W * lds_per_wave * sizeof(float) > 64 * 1024) W >>= 1;
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  const int64_t grid = (rows + W - 1) / W;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  hipLaunchKernelGGL((prefill_search_rows_kernel<T, D>), dim3((unsigned)grid), dim3(256),
                     (size_t)W * lds_per_wave * sizeof(float), st, static_cast<const T*>(Qs),
                     static_cast<const T*>(K), static_cast<const T*>(Ks), idx, scores, pb.Lq,
                     pb.q_pos0, pb.Hq, pb.G, pb.S, pb.topk, pb.n, W, lds_per_wave, pb.qsh, pb.qst,
                     pb.kvsh, pb.kvst);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

#define SL_DISPATCH(FN, ...)                                                   \
  do {                                                                         \
    if (pb.dtype == SL_BF16) {                                                 \
      if (pb.D == 128) return FN<bf16_t, 128>(__VA_ARGS__);                    \
      return FN<bf16_t, 64>(__VA_ARGS__);                                      \
    }                                                                          \
    if (pb.D == 128) return FN<float, 128>(__VA_ARGS__);                       \
    return FN<float, 64>(__VA_ARGS__);                                         \
  } while (0)

}  // namespace

// The selecting wavefront keeps one head's (decode) or one row's (prefill) scores in LDS.
constexpr int64_t kMaxSpansLds = 12288;

sl_status span_keys(const Problem& pb, const void* K, void* Ks, hipStream_t st) {
  SL_DISPATCH(launch_span_keys, pb, K, Ks, st);
}

size_t decode_search_ws_bytes(const Problem&) { return 0; }

sl_status decode_search(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                        int32_t* idx, float* scores, void* /*ws*/, hipStream_t st) {
  if (pb.n > kMaxSpansLds) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_decode_search, pb, Qs, K, Ks, idx, scores, st);
}

sl_status prefill_search_rows(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                              int32_t* idx, float* scores, hipStream_t st) {
  if (pb.n > kMaxSpansLds) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_prefill_search_rows, pb, Qs, K, Ks, idx, scores, st);
}

}  // namespace sl
