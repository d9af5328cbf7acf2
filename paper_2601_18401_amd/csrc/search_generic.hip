// Span-search kernels that need no matrix cores: the span-key gather, the decode form
// (one workgroup per head scores its candidates into LDS and selects) and the
// row-stationary prefill form (one wavefront per query row) used for fp32 and for shapes the
// MFMA path does not cover.
//
// Scores are eq. (2): raw dot products, accumulated in fp32 from exact products.
#include <cmath>

#include "kernels.h"
#include "select.h"

namespace sl {

int64_t decode_score_ld(const Problem& pb);

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
__device__ __forceinline__ void decode_search_body(
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
  const uint4 qraw = load16(Qs + (int64_t)h * qsh + lr * EPL);
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
      float acc = Piece<T>::dot(kr[u], qraw, 0.f);
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

template <typename T, int D>
__global__ __launch_bounds__(kDecodeSearchThreads) void decode_search_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, const T* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t c, int64_t n, int G, int S,
    int topk, int64_t qsh, int64_t kvsh, int64_t kvst) {
  decode_search_body<T, D>(Qs, K, Ks, idx, scores, c, n, G, S, topk, qsh, kvsh, kvst);
}

// Batched form (blockIdx.y = sequence); the dynamic LDS is sized for the longest sequence.
template <typename T, int D>
__global__ __launch_bounds__(kDecodeSearchThreads) void decode_search_batched_kernel(
    const sl_decode_seq* __restrict__ seqs, int G, int S, int topk, int64_t qsh, int64_t kvsh,
    int64_t kvst) {
  const sl_decode_seq sq = seqs[blockIdx.y];
  decode_search_body<T, D>(static_cast<const T*>(sq.Qs), static_cast<const T*>(sq.K),
                           static_cast<const T*>(sq.Ks), sq.idx, sq.scores, (sq.L - 1) / S,
                           (sq.L + S - 1) / S, G, S, topk, qsh, kvsh ? kvsh : sq.L * kvst, kvst);
}

// ------------------------------------------------------------------ a7: decode search, block-parallel select
// Same scoring as above, but the selection uses all 16 wavefronts and has no k-long chain of
// dependent rounds:
//   1. every thread owns up to RMAX consecutive candidates (registers);
//   2. the k-th largest value T is found by a most-significant-digit-first radix select on
//      order-preserving 32-bit keys: four passes of an 8-bit LDS histogram over the candidates
//      that still match the digits fixed so far; wavefront 0 picks the digit in which the k-th
//      largest key lies from a suffix sum over the 256 bins;
//   3. every candidate > T is selected, plus the lowest-index candidates == T that are needed to
//      reach k (ties to the lower index); the output slot of a selected candidate is the number
//      of selected candidates below it, from one block-wide prefix sum of (count > T, count == T).
template <typename T, int D, int RMAX>
__device__ __forceinline__ void decode_search_block_body(
    const T* __restrict__ Qs, const T* __restrict__ K, const T* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t c, int64_t n, int G, int S,
    int topk, int64_t qsh, int64_t kvsh, int64_t kvst, int64_t anchor_i, int anchor_s0,
    int anchor_root, const float* __restrict__ pre_scores = nullptr, int64_t pre_ld = 0) {
  // pre_scores: the head's candidate scores were computed by decode_score_group_kernel
  // (row h of a [Hq][pre_ld] array); the scoring loop is skipped.
  // anchor_i >= 0: the candidates are the anchors of query position anchor_i on the paper's
  // stride pattern (Section 3.3, p = 1/anchor_root): candidate j is stride index s = anchor_s0 + j
  // at token anchor_i - (s+1)^root + 1, its key is K at that token, and the output lists tokens.
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  constexpr int U = 16, NW = kDecodeSearchThreads / 64;
  auto anchor_token = [&](int64_t j) { return anchor_token_of(anchor_i, anchor_s0 + j, anchor_root); };
  __shared__ float s_sc[kDecodeSearchThreads * RMAX];
  __shared__ __align__(16) unsigned s_hist[4][256];  // one histogram per radix pass
  __shared__ int s_wave_tot[NW];
  const int h = blockIdx.x, kv = h / G;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  static_assert(kDecodeSearchThreads == 4 * 256, "one histogram bin per thread");
  s_hist[tid >> 8][tid & 255] = 0u;  // visible after the barrier that follows the scoring loop
  const int g = lane / LPR, lr = lane % LPR;
  const int kk = topk < c ? topk : (int)c;

  if (!pre_scores) {
    const uint4 qraw = load16(Qs + (int64_t)h * qsh + lr * EPL);
    for (int64_t jb = (int64_t)wave * RPW * U; jb < c; jb += NW * RPW * U) {
      uint4 kr[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        int64_t j = jb + u * RPW + g;
        j = j < c ? j : c - 1;
        const T* kp = anchor_i >= 0 ? K + kv * kvsh + anchor_token(j) * kvst
                                    : span_key_ptr<T, D>(K, Ks, kv, j, n, S, kvsh, kvst);
        kr[u] = load16(kp + lr * EPL);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float acc = Piece<T>::dot(kr[u], qraw, 0.f);
        acc = group_sum<LPR>(acc);
        const int64_t j = jb + u * RPW + g;
        if (lr == 0 && j < c) s_sc[j] = acc;
      }
    }
  }
  __syncthreads();  // the scores, and the cleared histograms

  // 1. thread t owns candidates t*R .. t*R + R-1 (index order = thread order)
  const int R = (int)((c + kDecodeSearchThreads - 1) / kDecodeSearchThreads);
  float v[RMAX];
  unsigned key[RMAX];
#pragma unroll
  for (int r = 0; r < RMAX; ++r) {
    const int j = tid * R + r;
    const bool in = r < R && j < c;
    v[r] = !in ? -INFINITY : pre_scores ? pre_scores[(int64_t)h * pre_ld + j] : s_sc[j];
    const unsigned u = __float_as_uint(v[r] + 0.0f);  // -0 scores as +0: equal scores, equal keys
    key[r] = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    if (!(v[r] > -INFINITY)) key[r] = 0u;  // empty slots (and non-finite input) never match
  }

  // 2. radix select of the kk-th largest key.  Tkey: every key above it is selected, keys equal to
  // it are ties (lowest index first).  The passes stop early when the bin that holds the kk-th
  // largest key is taken whole: every key at or above the bin's lower bound is then selected
  // (Tkey = that bound - 1; a valid key is never 0, so the bound is at least 1).
  unsigned Tkey = 0xffffffffu;  // kk == 0: nothing is selected
  if (kk > 0) {
    unsigned prefix = 0u, mask = 0u;
    int krem = kk;
    bool whole = false;
    for (int pass = 0; pass < 4 && !whole; ++pass) {
      const int shift = 24 - 8 * pass;
#pragma unroll
      for (int r = 0; r < RMAX; ++r)
        if (key[r] != 0u && (key[r] & mask) == prefix) atomicAdd(&s_hist[pass][(key[r] >> shift) & 255u], 1u);
      __syncthreads();
      // every wavefront finds the bin of the krem-th largest key by itself (one barrier per pass)
      const uint4 c4 = *reinterpret_cast<const uint4*>(&s_hist[pass][4 * lane]);
      const int lane_sum = (int)(c4.x + c4.y + c4.z + c4.w);
      const int incl = wave_inclusive_scan(lane_sum);
      const int total = __builtin_amdgcn_readlane(incl, 63);
      int above = total - incl;  // candidates in bins above this lane's four
      const unsigned cnt[4] = {c4.x, c4.y, c4.z, c4.w};
      int digit = -1, kleft = 0, inbin = 0;
#pragma unroll
      for (int b4 = 3; b4 >= 0; --b4) {
        if (above < krem && krem <= above + (int)cnt[b4]) {
          digit = 4 * lane + b4;
          kleft = krem - above;
          inbin = (int)cnt[b4];
        }
        above += (int)cnt[b4];
      }
      // exactly one lane holds the bin when 1 <= krem <= number of matching keys; NaN scores
      // (which never match) can leave none: bin 0 then, the result is unspecified but in bounds
      const unsigned long long found = __ballot(digit >= 0);
      const int src = found ? __builtin_ctzll(found) : 0;
      digit = found ? __builtin_amdgcn_readlane(digit, src) : 0;
      krem = found ? __builtin_amdgcn_readlane(kleft, src) : krem;
      whole = found && krem == __builtin_amdgcn_readlane(inbin, src);
      prefix |= (unsigned)digit << shift;
      mask |= 255u << shift;
    }
    Tkey = whole ? prefix - 1u : prefix;
  }

  // 3. select and place
  int gt = 0, eq = 0;
#pragma unroll
  for (int r = 0; r < RMAX; ++r) {
    gt += key[r] > Tkey ? 1 : 0;
    eq += (key[r] == Tkey && key[r] != 0u) ? 1 : 0;
  }
  const int packed = gt | (eq << 16);
  const int incl = wave_inclusive_scan(packed);
  if (lane == 63) s_wave_tot[wave] = incl;
  __syncthreads();
  int before = incl - packed, total = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const int t = s_wave_tot[w];
    before += w < wave ? t : 0;
    total += t;
  }
  const int gt_total = total & 0xffff;
  const int need_eq = kk - gt_total;  // ties accepted, lowest index first
  int gt_before = before & 0xffff, eq_before = before >> 16;
  int32_t* oi = idx + (int64_t)h * topk;
  float* os = scores ? scores + (int64_t)h * topk : nullptr;
#pragma unroll
  for (int r = 0; r < RMAX; ++r) {
    const bool is_gt = key[r] > Tkey;
    const bool is_eq = key[r] == Tkey && key[r] != 0u;
    if (is_gt || (is_eq && eq_before < need_eq)) {
      const int pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
      if ((unsigned)pos < (unsigned)kk) {  // always true unless scores are NaN
        oi[pos] = anchor_i >= 0 ? (int32_t)anchor_token(tid * R + r) : tid * R + r;
        if (os) os[pos] = v[r];
      }
    }
    gt_before += is_gt ? 1 : 0;
    eq_before += is_eq ? 1 : 0;
  }
  if (tid >= kk && tid < topk) {
    oi[tid] = -1;
    if (os) os[tid] = -INFINITY;
  }
}

template <typename T, int D, int RMAX>
__global__ __launch_bounds__(kDecodeSearchThreads) void decode_search_block_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, const T* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t c, int64_t n, int G, int S,
    int topk, int64_t qsh, int64_t kvsh, int64_t kvst, int64_t anchor_i, int anchor_s0,
    int anchor_root, const float* __restrict__ pre_scores, int64_t pre_ld) {
  decode_search_block_body<T, D, RMAX>(Qs, K, Ks, idx, scores, c, n, G, S, topk, qsh, kvsh, kvst,
                                       anchor_i, anchor_s0, anchor_root, pre_scores, pre_ld);
}

// First launch of the two-launch decode search: the candidates of a kv head are scored ONCE for
// all G query heads of its group, by many small workgroups (the key rows are read once instead
// of once per head, and from every compute unit instead of from Hq of them).  grid
// (ceil(c / kScoreCand), Hkv), 4 wavefronts; a wavefront takes kScoreCand / 4 consecutive
// candidates, LPR lanes per key row.  Same arithmetic as the one-launch kernel (Piece<T>::dot over
// the lane's elements, then the lane-group sum), so the scores are bit-identical to it.
constexpr int kScoreCand = 32;

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_score_group_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, const T* __restrict__ Ks,
    float* __restrict__ sc_out, int64_t c, int64_t n, int G, int S, int64_t qsh, int64_t kvsh,
    int64_t kvst, int64_t ld) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  constexpr int PER_WAVE = kScoreCand / 4, U = PER_WAVE / RPW;
  static_assert(U >= 1 && U * RPW == PER_WAVE, "candidates per wavefront must be whole load batches");
  const int kv = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane / LPR, lr = lane % LPR;
  const int64_t j0 = (int64_t)blockIdx.x * kScoreCand + wave * PER_WAVE;
  if (j0 >= c) return;
  uint4 kr[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t j = j0 + u * RPW + g;
    j = j < c ? j : c - 1;
    kr[u] = load16(span_key_ptr<T, D>(K, Ks, kv, j, n, S, kvsh, kvst) + lr * EPL);
  }
  constexpr int HB = 8;  // query heads per batch of query loads
  for (int h0 = 0; h0 < G; h0 += HB) {
    uint4 qr[HB];
#pragma unroll
    for (int b = 0; b < HB; ++b) {
      const int hh = kv * G + (h0 + b < G ? h0 + b : G - 1);
      qr[b] = load16(Qs + (int64_t)hh * qsh + lr * EPL);
    }
#pragma unroll
    for (int b = 0; b < HB; ++b) {
      const uint4 qraw = qr[b];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float acc = Piece<T>::dot(kr[u], qraw, 0.f);
        acc = group_sum<LPR>(acc);
        const int64_t j = j0 + u * RPW + g;
        if (lr == 0 && j < c && h0 + b < G) sc_out[(int64_t)(kv * G + h0 + b) * ld + j] = acc;
      }
    }
  }
}

// Batched decode: blockIdx.y is the sequence; candidates c = (L - 1) / S and the span-key row count
// n = ceil(L / S) follow from its own length.  kvsh = 0: the cache is packed for its own length.
template <typename T, int D, int RMAX>
__global__ __launch_bounds__(kDecodeSearchThreads) void decode_search_block_batched_kernel(
    const sl_decode_seq* __restrict__ seqs, int G, int S, int topk, int64_t qsh, int64_t kvsh,
    int64_t kvst) {
  const sl_decode_seq sq = seqs[blockIdx.y];
  decode_search_block_body<T, D, RMAX>(static_cast<const T*>(sq.Qs), static_cast<const T*>(sq.K),
                                       static_cast<const T*>(sq.Ks), sq.idx, sq.scores, (sq.L - 1) / S,
                                       (sq.L + S - 1) / S, G, S, topk, qsh, kvsh ? kvsh : sq.L * kvst,
                                       kvst, (int64_t)-1, 0, 2);
}

// Batched decode on the paper's geometry: every sequence has its own query position L - 1 and so
// its own candidate range (stride indices s0 .. s_max of that position).
template <typename T, int D, int RMAX>
__global__ __launch_bounds__(kDecodeSearchThreads) void anchor_search_block_batched_kernel(
    const sl_decode_seq* __restrict__ seqs, int G, int topk, int64_t qsh, int64_t kvsh, int64_t kvst,
    int64_t window, int root) {
  const sl_decode_seq sq = seqs[blockIdx.y];
  const int64_t i = sq.L - 1;
  const int64_t s_max = iroot_floor(i + 1, root) - 1;
  const int64_t first = window > 0 ? iroot_floor(window, root) : 0;
  const int64_t c = s_max >= first ? s_max - first + 1 : 0;
  decode_search_block_body<T, D, RMAX>(static_cast<const T*>(sq.Qs), static_cast<const T*>(sq.K),
                                       static_cast<const T*>(nullptr), sq.idx, sq.scores, c, (int64_t)0, G,
                                       1, topk, qsh, kvsh ? kvsh : sq.L * kvst, kvst, i, (int)first, root);
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
  const uint4 qraw = load16(Qs + h * qsh + r * qst + lr * EPL);
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
      float acc = Piece<T>::dot(kr[u], qraw, 0.f);
      acc = group_sum<LPR>(acc);
      const int64_t j = jb + u * RPW + g;
      if (lr == 0 && j < c) sc[lm.slot((int)j)] = acc;
    }
  }
  __builtin_amdgcn_wave_barrier();
  wave_select_topk(sc, lm, (int)c, topk, lane, idx + row * topk,
                   scores ? scores + row * topk : nullptr);
}

// The paper's geometry, prefill form, search (Section 3.3, Algorithm 1; eq. (2)-(3) with
// K_a = K): one wavefront per (head, query row).  The candidates of the query at position i are
// the anchors t_s = i - (s+1)^root + 1 with s0 <= s and t_s >= 0 (s0 = floor(window^(1/root)):
// anchors inside the window are left out); candidate number j is stride index s0 + j.
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_anchor_search_rows_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, int32_t* __restrict__ anchors,
    float* __restrict__ scores, int64_t Lq, int64_t q_pos0, int Hq, int G, int topk, int s0, int root,
    int W, int lds_per_wave, int64_t qsh, int64_t qst, int64_t kvsh, int64_t kvst) {
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
  const int64_t s_max = iroot_floor(i + 1, root) - 1;  // (s+1)^root <= i + 1
  const int64_t c = s_max >= s0 ? s_max - s0 + 1 : 0;
  const int g = lane / LPR, lr = lane % LPR;
  const LaneMajor lm = LaneMajor::make(c);
  select_clear(sc, lm, lane);
  __builtin_amdgcn_wave_barrier();
  const uint4 qraw = load16(Qs + h * qsh + r * qst + lr * EPL);
  const T* Kb = K + kv * kvsh;
  constexpr int U = 4;
  for (int64_t jb = 0; jb < c; jb += RPW * U) {
    uint4 kr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t j = jb + u * RPW + g;
      j = j < c ? j : c - 1;
      kr[u] = load16(Kb + anchor_token_of(i, s0 + j, root) * kvst + lr * EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float acc = Piece<T>::dot(kr[u], qraw, 0.f);
      acc = group_sum<LPR>(acc);
      const int64_t j = jb + u * RPW + g;
      if (lr == 0 && j < c) sc[lm.slot((int)j)] = acc;
    }
  }
  __builtin_amdgcn_wave_barrier();
  wave_select_topk(sc, lm, (int)c, topk, lane, anchors + row * topk,
                   scores ? scores + row * topk : nullptr, i, s0, root);
}

// The same search with the key rows shared by the query heads of a kv group: a row group of LPR
// lanes owns one query row and up to 8 query heads of its kv head; every candidate's key row is
// loaded once and scored against all of them (the row-per-wavefront kernel above loads it once per
// head: 8x the L2 traffic at GQA 8:1, which is what bounds it).  Lane lr of a group keeps the
// running top-KMAX (scores and candidate numbers, in registers) of head lr % 8; candidates come in
// ascending stride index and only a strictly larger score displaces an entry, so ties stay with the
// nearer anchor.  Arithmetic per score as everywhere else (Piece<T>::dot over the lane's
// elements, then the lane-group sum): bit-identical to the other search kernels.
template <typename T, int D, int KMAX>
__global__ __launch_bounds__(256) void prefill_anchor_search_group_kernel(
    const T* __restrict__ Qs, const T* __restrict__ K, int32_t* __restrict__ anchors,
    float* __restrict__ scores, int64_t Lq, int64_t q_pos0, int G, int topk, int s0, int root,
    int64_t qsh, int64_t qst, int64_t kvsh, int64_t kvst) {
  using RL = RowLayout<T, D>;
  constexpr int EPL = RL::EPL, LPR = RL::LPR, RPW = RL::RPW;
  constexpr int HB = 8, U = 8;
  static_assert(LPR >= HB, "a row group needs a lane per head of the batch");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane / LPR, lr = lane % LPR;
  const int nb = (G + HB - 1) / HB;
  const int kv = blockIdx.y / nb, h0 = (blockIdx.y % nb) * HB;
  const int64_t r = ((int64_t)blockIdx.x * 4 + wave) * RPW + g;
  if (((int64_t)blockIdx.x * 4 + wave) * RPW >= Lq) return;  // the whole wavefront is past the last row
  const int64_t rc = r < Lq ? r : Lq - 1;
  const int64_t i = q_pos0 + rc;
  const int64_t s_max = iroot_floor(i + 1, root) - 1;  // (s+1)^root <= i + 1
  const int c = s_max >= s0 ? (int)(s_max - s0 + 1) : 0;
  // rows ascend with the lane and so do their candidate counts: the last lane has the most
  const int c_wave = __builtin_amdgcn_readlane(c, 63);

  uint4 qraw[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    const int h = kv * G + (h0 + hb < G ? h0 + hb : G - 1);
    qraw[hb] = load16(Qs + h * qsh + rc * qst + lr * EPL);
  }
  const T* Kb = K + kv * kvsh;
  float v[KMAX];
  int id[KMAX];
#pragma unroll
  for (int e = 0; e < KMAX; ++e) {
    v[e] = -INFINITY;
    id[e] = -1;
  }
  const int myh = lr % HB;
  for (int jb = 0; jb < c_wave; jb += U) {
    uint4 kr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = jb + u < c ? jb + u : c - 1;
      const int64_t t = c > 0 ? anchor_token_of(i, (int64_t)s0 + j, root) : i;  // no candidate: any valid row
      kr[u] = load16(Kb + t * kvst + lr * EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // the eight heads' partial dot products, then one reduce-scatter: this lane gets head myh's score
      float part[HB];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) part[hb] = Piece<T>::dot(kr[u], qraw[hb], 0.f);
      float x = group_sum_scatter8<LPR>(part, lr);
      const int j = jb + u;
      x = j < c ? x : -INFINITY;
      // insert (x, j): slot e takes the entry above it if x belongs above that one, x itself if
      // x belongs exactly here; strict compares keep the earlier candidate on ties
#pragma unroll
      for (int e = KMAX - 1; e >= 0; --e) {
        const bool up = e > 0 && x > v[e > 0 ? e - 1 : 0];
        const bool here = !up && x > v[e];
        id[e] = up ? id[e > 0 ? e - 1 : 0] : (here ? j : id[e]);
        v[e] = up ? v[e > 0 ? e - 1 : 0] : (here ? x : v[e]);
      }
    }
  }
  if (r < Lq && lr < HB && h0 + lr < G) {
    const int64_t row = (int64_t)(kv * G + h0 + lr) * Lq + r;
    int32_t* oa = anchors + row * topk;
    float* os = scores ? scores + row * topk : nullptr;
    int kk = 0;
#pragma unroll
    for (int e = 0; e < KMAX; ++e) kk += (e < topk && id[e] >= 0) ? 1 : 0;
    // nearest anchor first: a selected entry's slot is the number of selected entries with a lower stride index
#pragma unroll
    for (int e = 0; e < KMAX; ++e) {
      if (e < topk && id[e] >= 0) {
        int rank = 0;
#pragma unroll
        for (int e2 = 0; e2 < KMAX; ++e2) rank += (e2 < topk && id[e2] >= 0 && id[e2] < id[e]) ? 1 : 0;
        oa[rank] = (int32_t)anchor_token_of(i, (int64_t)s0 + id[e], root);
        if (os) os[rank] = v[e];
      }
    }
    for (int e = kk; e < topk; ++e) {
      oa[e] = -1;
      if (os) os[e] = -INFINITY;
    }
  }
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
                               int32_t* idx, float* scores, void* ws, hipStream_t st) {
  const int64_t c = pb.q_pos0 / pb.S;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  if (c <= (int64_t)kDecodeSearchThreads * 4) {
    // Two launches: the group-wide scoring kernel fills the workspace [Hq][ld], then one workgroup
    // per head selects (block-parallel selection: candidates fit 4 registers per thread).
    // (a cache with more spans than that sizes no workspace: its shorter queries score in the
    // selecting workgroup itself)
    float* sc_ws = pb.n <= (int64_t)kDecodeSearchThreads * 4 ? static_cast<float*>(ws) : nullptr;
    const int64_t ld = decode_score_ld(pb);
    if (c > 0 && sc_ws)
      hipLaunchKernelGGL((decode_score_group_kernel<T, D>), dim3((unsigned)((c + kScoreCand - 1) / kScoreCand), pb.Hkv),
                         dim3(256), 0, st, static_cast<const T*>(Qs), static_cast<const T*>(K),
                         static_cast<const T*>(Ks), sc_ws, c, pb.n, pb.G, pb.S, pb.qsh, pb.kvsh, pb.kvst, ld);
    if (c <= kDecodeSearchThreads)
      hipLaunchKernelGGL((decode_search_block_kernel<T, D, 1>), dim3(pb.Hq),
                         dim3(kDecodeSearchThreads), 0, st, static_cast<const T*>(Qs),
                         static_cast<const T*>(K), static_cast<const T*>(Ks), idx, scores, c, pb.n,
                         pb.G, pb.S, pb.topk, pb.qsh, pb.kvsh, pb.kvst, (int64_t)-1, 0, 2, sc_ws, ld);
    else
      hipLaunchKernelGGL((decode_search_block_kernel<T, D, 4>), dim3(pb.Hq),
                         dim3(kDecodeSearchThreads), 0, st, static_cast<const T*>(Qs),
                         static_cast<const T*>(K), static_cast<const T*>(Ks), idx, scores, c, pb.n,
                         pb.G, pb.S, pb.topk, pb.qsh, pb.kvsh, pb.kvst, (int64_t)-1, 0, 2, sc_ws, ld);
    if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
  }
  hipLaunchKernelGGL((decode_search_kernel<T, D>), dim3(pb.Hq), dim3(kDecodeSearchThreads),
                     (size_t)LaneMajor::make(c).lds_floats() * sizeof(float), st,
                     static_cast<const T*>(Qs),
                     static_cast<const T*>(K), static_cast<const T*>(Ks), idx, scores, c, pb.n,
                     pb.G, pb.S, pb.topk, pb.qsh, pb.kvsh, pb.kvst);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_decode_search_batched(const Problem& pb, const sl_decode_seq* seqs, int B,
                                       hipStream_t st) {
  const int64_t c_max = pb.q_pos0 / pb.S;  // of the longest sequence
  const int64_t kvsh = pb.kvsh_given ? pb.kvsh : 0;
  if (c_max > (int64_t)kDecodeSearchThreads * 4)
    hipLaunchKernelGGL((decode_search_batched_kernel<T, D>), dim3(pb.Hq, B), dim3(kDecodeSearchThreads),
                       (size_t)LaneMajor::make(c_max).lds_floats() * sizeof(float), st, seqs, pb.G, pb.S,
                       pb.topk, pb.qsh, kvsh, pb.kvst);
  else if (c_max <= kDecodeSearchThreads)
    hipLaunchKernelGGL((decode_search_block_batched_kernel<T, D, 1>), dim3(pb.Hq, B),
                       dim3(kDecodeSearchThreads), 0, st, seqs, pb.G, pb.S, pb.topk, pb.qsh, kvsh,
                       pb.kvst);
  else
    hipLaunchKernelGGL((decode_search_block_batched_kernel<T, D, 4>), dim3(pb.Hq, B),
                       dim3(kDecodeSearchThreads), 0, st, seqs, pb.G, pb.S, pb.topk, pb.qsh, kvsh,
                       pb.kvst);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_anchor_search_batched(const Problem& pb, const sl_decode_seq* seqs, int B, int64_t c_max,
                                       int64_t window, int root, hipStream_t st) {
  const int64_t kvsh = pb.kvsh_given ? pb.kvsh : 0;
  if (c_max <= kDecodeSearchThreads)
    hipLaunchKernelGGL((anchor_search_block_batched_kernel<T, D, 1>), dim3(pb.Hq, B),
                       dim3(kDecodeSearchThreads), 0, st, seqs, pb.G, pb.topk, pb.qsh, kvsh, pb.kvst,
                       window, root);
  else
    hipLaunchKernelGGL((anchor_search_block_batched_kernel<T, D, 4>), dim3(pb.Hq, B),
                       dim3(kDecodeSearchThreads), 0, st, seqs, pb.G, pb.topk, pb.qsh, kvsh, pb.kvst,
                       window, root);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

template <typename T, int D>
sl_status launch_anchor_search(const Problem& pb, const void* Qs, const void* K, int32_t* anchors,
                               float* scores, int64_t c, int s0, int root, hipStream_t st) {
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  if (c <= kDecodeSearchThreads)
    hipLaunchKernelGGL((decode_search_block_kernel<T, D, 1>), dim3(pb.Hq), dim3(kDecodeSearchThreads),
                       0, st, static_cast<const T*>(Qs), static_cast<const T*>(K),
                       static_cast<const T*>(nullptr), anchors, scores, c, (int64_t)0, pb.G, 1,
                       pb.topk, pb.qsh, pb.kvsh, pb.kvst, pb.q_pos0, s0, root,
                       static_cast<const float*>(nullptr), (int64_t)0);
  else
    hipLaunchKernelGGL((decode_search_block_kernel<T, D, 4>), dim3(pb.Hq), dim3(kDecodeSearchThreads),
                       0, st, static_cast<const T*>(Qs), static_cast<const T*>(K),
                       static_cast<const T*>(nullptr), anchors, scores, c, (int64_t)0, pb.G, 1,
                       pb.topk, pb.qsh, pb.kvsh, pb.kvst, pb.q_pos0, s0, root,
                       static_cast<const float*>(nullptr), (int64_t)0);
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

template <typename T, int D>
sl_status launch_anchor_search_rows(const Problem& pb, const void* Qs, const void* K,
                                    int32_t* anchors, float* scores, int64_t c_max, int s0,
                                    int root, hipStream_t st) {
  if (pb.topk <= 8) {  // key rows shared by the heads of a kv group, top-k lists in registers
    constexpr int RPW = RowLayout<T, D>::RPW;
    const dim3 grid((unsigned)((pb.Lq + 4 * RPW - 1) / (4 * RPW)), (unsigned)(pb.Hkv * ((pb.G + 7) / 8)));
    if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
#define SL_ANCHOR_GROUP(KM)                                                                               \
  hipLaunchKernelGGL((prefill_anchor_search_group_kernel<T, D, KM>), grid, dim3(256), 0, st,              \
                     static_cast<const T*>(Qs), static_cast<const T*>(K), anchors, scores, pb.Lq, pb.q_pos0, \
                     pb.G, pb.topk, s0, root, pb.qsh, pb.qst, pb.kvsh, pb.kvst)
    if (pb.topk <= 2) SL_ANCHOR_GROUP(2);
    else if (pb.topk <= 4) SL_ANCHOR_GROUP(4);
    else SL_ANCHOR_GROUP(8);
#undef SL_ANCHOR_GROUP
    if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
  }
  const int lds_per_wave = LaneMajor::make(c_max).lds_floats();
  int W = 4;
  while (W > 1 && (size_t)W * lds_per_wave * sizeof(float) > 64 * 1024) W >>= 1;
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  const int64_t grid = (rows + W - 1) / W;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  hipLaunchKernelGGL((prefill_anchor_search_rows_kernel<T, D>), dim3((unsigned)grid), dim3(256),
                     (size_t)W * lds_per_wave * sizeof(float), st, static_cast<const T*>(Qs),
                     static_cast<const T*>(K), anchors, scores, pb.Lq, pb.q_pos0, pb.Hq, pb.G,
                     pb.topk, s0, root, W, lds_per_wave, pb.qsh, pb.qst, pb.kvsh, pb.kvst);
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

// Row length (floats) of the decode search's score workspace [Hq][ld]: the candidate spans,
// rounded up to whole 256-byte lines.
int64_t decode_score_ld(const Problem& pb) { return (int64_t)align_up((size_t)(pb.n > 0 ? pb.n : 1), 64); }

size_t decode_search_ws_bytes(const Problem& pb) {
  // more candidates than the block-parallel selection takes: the one-launch kernel, no workspace
  if (pb.n > (int64_t)kDecodeSearchThreads * 4) return 0;
  return (size_t)pb.Hq * decode_score_ld(pb) * sizeof(float);
}

// Candidate anchors of query position i = pb.q_pos0 with window w (Section 3.3, Algorithm 1):
// stride indices s0 .. s_max, where t_s = i - (s+1)^root + 1 >= 0 and t_s < i - w + 1.
void anchor_candidates(const Problem& pb, int64_t window, int root, int64_t* c, int* s0) {
  const int64_t i = pb.q_pos0;
  const int64_t s_max = iroot_floor(i + 1, root) - 1;               // (s+1)^root <= i + 1
  const int64_t first = window > 0 ? iroot_floor(window, root) : 0;  // (s+1)^root > w  <=>  s >= floor(w^(1/root))
  *s0 = (int)first;
  *c = s_max >= first ? s_max - first + 1 : 0;
}

sl_status anchor_search_decode(const Problem& pb, int64_t window, int root, const void* Qs,
                               const void* K, int32_t* anchors, float* scores, hipStream_t st) {
  int64_t c;
  int s0;
  anchor_candidates(pb, window, root, &c, &s0);
  if (c > (int64_t)kDecodeSearchThreads * 4) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_anchor_search, pb, Qs, K, anchors, scores, c, s0, root, st);
}

sl_status anchor_search_prefill(const Problem& pb, int64_t window, int root, const void* Qs,
                                const void* K, int32_t* anchors, float* scores, hipStream_t st) {
  // the last query row has the most candidates
  Problem last = pb;
  last.q_pos0 = pb.q_pos0 + pb.Lq - 1;
  int64_t c_max;
  int s0;
  anchor_candidates(last, window, root, &c_max, &s0);
  if (c_max > kMaxSpansLds) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_anchor_search_rows, pb, Qs, K, anchors, scores, c_max, s0, root, st);
}

sl_status anchor_search_decode_batched(const Problem& pb, int64_t window, int root,
                                       const sl_decode_seq* seqs, int B, hipStream_t st) {
  int64_t c_max;  // of the longest sequence: candidates only grow with the position
  int s0;
  anchor_candidates(pb, window, root, &c_max, &s0);
  if (c_max > (int64_t)kDecodeSearchThreads * 4) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_anchor_search_batched, pb, seqs, B, c_max, window, root, st);
}

sl_status decode_search_batched(const Problem& pb, const sl_decode_seq* seqs, int B, hipStream_t st) {
  if (pb.n > kMaxSpansLds) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_decode_search_batched, pb, seqs, B, st);
}

sl_status decode_search(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                        int32_t* idx, float* scores, void* ws, hipStream_t st) {
  if (pb.n > kMaxSpansLds) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_decode_search, pb, Qs, K, Ks, idx, scores, ws, st);
}

sl_status prefill_search_rows(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                              int32_t* idx, float* scores, hipStream_t st) {
  if (pb.n > kMaxSpansLds) return SL_ERR_UNSUPPORTED;
  SL_DISPATCH(launch_prefill_search_rows, pb, Qs, K, Ks, idx, scores, st);
}

}  // namespace sl
