// Prefill span-search on the matrix cores (bf16, D = 128).
//
// Scores (eq. (2)) are computed transposed, S^T[span][query] = Ks[span][:] . Qs[query][:], so
// that after v_mfma_f32_32x32x16_bf16 a lane owns one query column: lane l holds query l%32 and
// the 16 spans 8*(r/4) + 4*(l/32) + r%4 of a 32-span tile.  Each lane keeps the running top-k
// (eq. (3)) of the spans it sees; the selection itself is a threshold found in a first pass and
// applied in a second one (see the kernel).  Scores never leave the chip.
//
// Ties: among the spans whose score equals the threshold, the lower indices are kept.
#include "kernels.h"

namespace sl {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int HD = 128;
constexpr int TMQ = 128;        // query rows per workgroup (4 wavefronts x 32 columns)
constexpr int TNS = 64;         // span keys per staged chunk
constexpr int KSTR = HD + 8;    // LDS row stride (bf16 elements): conflict-free 16-byte reads
constexpr int kEmpty = 0x7fffffff;

// Running top-K VALUES of the candidates a lane has seen, sorted descending.  Inserting x is one
// median-of-three per slot: new v[e] = med3(x, v[e-1], v[e]) (x above v[e-1]: v[e-1] moves down;
// x between: x lands here; x below v[e]: unchanged), and v[0] = max(x, v[0]).
template <int KMAX>
struct TopVals {
  float v[KMAX];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int e = 0; e < KMAX; ++e) v[e] = -INFINITY;
  }
  __device__ __forceinline__ void push(float x) {
#pragma unroll
    for (int e = KMAX - 1; e >= 1; --e) v[e] = __builtin_amdgcn_fmed3f(x, v[e - 1], v[e]);
    v[0] = fmaxf(x, v[0]);
  }
};

// Two passes over the candidate spans of 128 query rows (4 wavefronts x 32 columns):
//   pass 1  keeps, per lane, only the VALUES of the top-k scores it has seen (a lane sees half of
//           its column's spans); the two lanes of a column are merged at the end, which gives the
//           column's threshold T = k'-th largest score, k' = min(topk, c), and the number of
//           scores above it;
//   pass 2  recomputes the scores (the MFMAs are cheap next to the selection arithmetic) and
//           appends every span with score > T, and up to need = k' - #(> T) spans per lane with
//           score == T (its lowest-index ones), to the column's list in LDS;
//   finish  one lane per column keeps the spans above T plus the `need` lowest-index spans at T
//           (ties go to the lower index), and writes them in ascending span order.
// Tracking values only makes the per-candidate cost of pass 1 k median instructions instead of
// the compare-and-select chains that carrying the indices along would need.
// WS: the scores of the selected spans are written too (their list costs LDS, which limits the
// resident workgroups; most callers only want the indices).
// The kernel is bound by the latency of its stages (two barriers and a global -> register -> LDS
// hand-over per 64 span keys), so resident workgroups count: without the score list and with
// topk <= 8 the registers are capped at 128 for a fourth workgroup per compute unit (-8 % at 256K
// tokens, -14 % at 64K; a fifth would spill).
template <int KMAX, bool WS>
__global__ __launch_bounds__(256, (KMAX == 8 && !WS) ? 4 : 1) void prefill_search_mfma_kernel(
    const bf16_t* __restrict__ Qs, const bf16_t* __restrict__ K, const bf16_t* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t Lq, int64_t q_pos0, int G, int S,
    int topk, int64_t n, int64_t qsh, int64_t qst, int64_t kvsh, int64_t kvst) {
  constexpr int CAP = 3 * KMAX;  // list entries per column: < KMAX above T, <= KMAX at T from each lane
  __shared__ __align__(16) bf16_t s_k[TNS * KSTR];
  __shared__ int s_cnt[TMQ];
  __shared__ int s_j[TMQ][CAP + 1];  // odd row stride: the lanes of a wavefront read their own rows
  __shared__ float s_x[WS ? TMQ : 1][CAP + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qc = lane & 31, hf = lane >> 5;
  const int col = wave * 32 + qc;
  const int tiles_per_head = (int)((Lq + TMQ - 1) / TMQ);
  const int h = blockIdx.x / tiles_per_head;
  const int64_t r0 = (int64_t)(blockIdx.x % tiles_per_head) * TMQ;
  const int kv = h / G;
  const int64_t r = r0 + col;
  const int64_t rc = r < Lq ? r : Lq - 1;
  const int c_q = (int)((q_pos0 + rc) / S);  // candidates of this lane's query: spans [0, c_q)
  const int64_t r_last = (r0 + TMQ - 1 < Lq ? r0 + TMQ - 1 : Lq - 1);
  const int c_max = (int)((q_pos0 + r_last) / S);
  const int c_lo = __builtin_amdgcn_readfirstlane(c_q);  // rows ascend with the lane: lane 0 has the lowest c
  if (tid < TMQ) s_cnt[tid] = 0;

  bf16x8 qf[8];
  {
    const bf16_t* qp = Qs + h * qsh + rc * qst;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + hf * 8);
  }

  // Walks the candidate spans in tiles of 32 and hands the lane's 16 scores of a tile, in
  // ascending span order, to f(score, span index); scores of spans >= c_q come as -inf.
  auto for_each_candidate = [&](auto f) {
    // 64 span keys per stage, 16 lanes x 16 bytes per key; the next stage's keys are fetched into
    // registers while the current stage is scored
    uint4 pre[4];
    auto fetch = [&](int j0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int id = tid + 256 * i, row = id >> 4, piece = id & 15;
        int64_t j = j0 + row;
        j = j < c_max ? j : c_max - 1;
        const bf16_t* src = Ks ? Ks + ((int64_t)kv * n + j) * HD : K + kv * kvsh + ((j + 1) * S - 1) * kvst;
        pre[i] = load16(src + piece * 8);
      }
    };
    if (c_max > 0) fetch(0);
    for (int j0 = 0; j0 < c_max; j0 += TNS) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int id = tid + 256 * i, row = id >> 4, piece = id & 15;
        *reinterpret_cast<uint4*>(&s_k[row * KSTR + piece * 8]) = pre[i];
      }
      __syncthreads();
      if (j0 + TNS < c_max) fetch(j0 + TNS);
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        if (j0 + 32 * sub < c_max) {  // uniform over the workgroup
          f32x16 s;
#pragma unroll
          for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
          for (int kk = 0; kk < 8; ++kk) {
            const bf16x8 ka =
                *reinterpret_cast<const bf16x8*>(&s_k[(32 * sub + qc) * KSTR + kk * 16 + hf * 8]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[kk], s, 0, 0, 0);
          }
          // causal: only complete spans below the query's own.  A tile that ends at or below the
          // lowest c of the wavefront (its first column's) needs no masking.
          if (j0 + 32 * sub + 32 <= c_lo) {
#pragma unroll
            for (int e = 0; e < 16; ++e) f(s[e], j0 + 32 * sub + 8 * (e >> 2) + 4 * hf + (e & 3));
          } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int j = j0 + 32 * sub + 8 * (e >> 2) + 4 * hf + (e & 3);
              f(j < c_q ? s[e] : -INFINITY, j);
            }
          }
        }
      }
      __syncthreads();
    }
  };

  // ---- pass 1: the column's top-k values
  TopVals<KMAX> top;
  top.init();
  for_each_candidate([&](float x, int) { top.push(x); });
  {
    float pv[KMAX];
#pragma unroll
    for (int e = 0; e < KMAX; ++e) {
      // the two results are {own, partner} in an order that depends on the lane half: take
      // the one that is not this lane's own (if both are equal either will do)
      const int own = __float_as_int(top.v[e]);
      auto a = __builtin_amdgcn_permlane32_swap(own, own, false, false);
      pv[e] = __int_as_float(a[0] == own ? a[1] : a[0]);
    }
#pragma unroll
    for (int e = 0; e < KMAX; ++e) top.push(pv[e]);
  }
  const int kq = topk < c_q ? topk : c_q;  // spans to select for this column
  float thr = INFINITY;                    // kq == 0: nothing passes
  int n_gt = 0;
#pragma unroll
  for (int e = 0; e < KMAX; ++e) thr = (e == kq - 1) ? top.v[e] : thr;
#pragma unroll
  for (int e = 0; e < KMAX; ++e) n_gt += (e < kq && top.v[e] > thr) ? 1 : 0;
  const int need_eq = kq - n_gt;           // >= 1 when kq >= 1

  // ---- pass 2: collect the spans at or above the threshold
  int n_eq = 0;  // spans at the threshold this lane has listed
  for_each_candidate([&](float x, int j) {
    if (x >= thr) {  // rare: at most k' + ties of the column's candidates
      const bool eq = x == thr;
      if (!eq || n_eq < need_eq) {
        const int pos = atomicAdd(&s_cnt[col], 1);
        s_j[col][pos] = eq ? (j | 0x40000000) : j;
        if (WS) s_x[col][pos] = x;
        n_eq += eq ? 1 : 0;
      }
    }
  });
  __syncthreads();

  // ---- finish: the column's two lanes share its list entries.  An entry at the threshold is
  // kept if fewer than need_eq such entries have a lower index; the kept ones below an entry are
  // then the entries above the threshold plus min(#at-threshold below it, need_eq).
  if (r < Lq) {
    const int cnt = s_cnt[col];
    int32_t* oi = idx + ((int64_t)h * Lq + r) * topk;
    float* os = WS ? scores + ((int64_t)h * Lq + r) * topk : nullptr;
    for (int u = hf; u < cnt; u += 2) {
      const int eu = s_j[col][u], ju = eu & 0x3fffffff;
      int lower_gt = 0, lower_eq = 0;
      for (int w = 0; w < cnt; ++w) {
        const int ew = s_j[col][w];
        const bool below = (ew & 0x3fffffff) < ju;
        lower_eq += (below && (ew & 0x40000000) != 0) ? 1 : 0;
        lower_gt += (below && (ew & 0x40000000) == 0) ? 1 : 0;
      }
      if ((eu & 0x40000000) == 0 || lower_eq < need_eq) {
        const int rank = lower_gt + (lower_eq < need_eq ? lower_eq : need_eq);
        oi[rank] = ju;
        if (WS) os[rank] = s_x[col][u];
      }
    }
  }
  if (hf == 0 && r < Lq) {
    int32_t* oi = idx + ((int64_t)h * Lq + r) * topk;
    float* os = WS ? scores + ((int64_t)h * Lq + r) * topk : nullptr;
    for (int e = kq; e < topk; ++e) {
      oi[e] = -1;
      if (os) os[e] = -INFINITY;
    }
  }
}

template <int KMAX>
sl_status launch(const Problem& pb, const void* Qs, const void* K, const void* Ks, int32_t* idx,
                 float* scores, hipStream_t st) {
  const int tiles_per_head = (int)((pb.Lq + TMQ - 1) / TMQ);
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  if (scores)
    hipLaunchKernelGGL((prefill_search_mfma_kernel<KMAX, true>), dim3(pb.Hq * tiles_per_head), dim3(256),
                       0, st, static_cast<const bf16_t*>(Qs), static_cast<const bf16_t*>(K),
                       static_cast<const bf16_t*>(Ks), idx, scores, pb.Lq, pb.q_pos0, pb.G, pb.S,
                       pb.topk, pb.n, pb.qsh, pb.qst, pb.kvsh, pb.kvst);
  else
    hipLaunchKernelGGL((prefill_search_mfma_kernel<KMAX, false>), dim3(pb.Hq * tiles_per_head), dim3(256),
                       0, st, static_cast<const bf16_t*>(Qs), static_cast<const bf16_t*>(K),
                       static_cast<const bf16_t*>(Ks), idx, scores, pb.Lq, pb.q_pos0, pb.G, pb.S,
                       pb.topk, pb.n, pb.qsh, pb.qst, pb.kvsh, pb.kvst);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

}  // namespace

bool prefill_search_mfma_supported(const Problem& pb) {
  return pb.dtype == SL_BF16 && pb.D == HD && (int64_t)pb.Hq * ((pb.Lq + TMQ - 1) / TMQ) < ((int64_t)1 << 31);
}

sl_status prefill_search_mfma(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                              int32_t* idx, float* scores, hipStream_t st) {
  if (pb.topk <= 8) return launch<8>(pb, Qs, K, Ks, idx, scores, st);
  if (pb.topk <= 16) return launch<16>(pb, Qs, K, Ks, idx, scores, st);
  return launch<32>(pb, Qs, K, Ks, idx, scores, st);
}

}  // namespace sl
