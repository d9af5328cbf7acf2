// Prefill span-search on the matrix cores (bf16, D = 128).
//
// Scores (eq. (2)) are computed transposed, S^T[span][query] = Ks[span][:] . Qs[query][:], so
// that after v_mfma_f32_32x32x16_bf16 a lane owns one query column: lane l holds query l%32 and
// the 16 spans 8*(r/4) + 4*(l/32) + r%4 of a 32-span tile.  Each lane keeps the running top-k
// (eq. (3)) of the spans it sees as a sorted list in registers; the two lanes of a column are
// merged at the end.  Scores never leave the chip.
//
// Ties: a lane meets its candidates in ascending span index and inserts on strict '>' only, so
// the earlier (lower) index stays ahead; the final merge of the two lanes compares (score, index).
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

template <int KMAX>
struct TopList {
  float v[KMAX];
  int j[KMAX];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int e = 0; e < KMAX; ++e) {
      v[e] = -INFINITY;
      j[e] = kEmpty;
    }
  }
  // insert a candidate that arrives in ascending index order: strict compare on the score
  __device__ __forceinline__ void push(float x, int xj) {
    bool gt[KMAX];
#pragma unroll
    for (int e = 0; e < KMAX; ++e) gt[e] = x > v[e];
#pragma unroll
    for (int e = KMAX - 1; e >= 1; --e) {
      v[e] = gt[e - 1] ? v[e - 1] : (gt[e] ? x : v[e]);
      j[e] = gt[e - 1] ? j[e - 1] : (gt[e] ? xj : j[e]);
    }
    v[0] = gt[0] ? x : v[0];
    j[0] = gt[0] ? xj : j[0];
  }
  // insert an arbitrary candidate: order by (score desc, index asc)
  __device__ __forceinline__ void push_any(float x, int xj) {
    bool gt[KMAX];
#pragma unroll
    for (int e = 0; e < KMAX; ++e) gt[e] = x > v[e] || (x == v[e] && xj < j[e]);
#pragma unroll
    for (int e = KMAX - 1; e >= 1; --e) {
      v[e] = gt[e - 1] ? v[e - 1] : (gt[e] ? x : v[e]);
      j[e] = gt[e - 1] ? j[e - 1] : (gt[e] ? xj : j[e]);
    }
    v[0] = gt[0] ? x : v[0];
    j[0] = gt[0] ? xj : j[0];
  }
};

template <int KMAX>
__global__ __launch_bounds__(256) void prefill_search_mfma_kernel(
    const bf16_t* __restrict__ Qs, const bf16_t* __restrict__ K, const bf16_t* __restrict__ Ks,
    int32_t* __restrict__ idx, float* __restrict__ scores, int64_t Lq, int64_t q_pos0, int G, int S,
    int topk, int64_t n, int64_t qsh, int64_t qst, int64_t kvsh, int64_t kvst) {
  __shared__ __align__(16) bf16_t s_k[TNS * KSTR];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qc = lane & 31, hf = lane >> 5;
  const int tiles_per_head = (int)((Lq + TMQ - 1) / TMQ);
  const int h = blockIdx.x / tiles_per_head;
  const int64_t r0 = (int64_t)(blockIdx.x % tiles_per_head) * TMQ;
  const int kv = h / G;
  const int64_t r = r0 + wave * 32 + qc;
  const int64_t rc = r < Lq ? r : Lq - 1;
  const int c_q = (int)((q_pos0 + rc) / S);  // candidates of this lane's query: spans [0, c_q)
  const int64_t r_last = (r0 + TMQ - 1 < Lq ? r0 + TMQ - 1 : Lq - 1);
  const int c_max = (int)((q_pos0 + r_last) / S);

  bf16x8 qf[8];
  {
    const bf16_t* qp = Qs + h * qsh + rc * qst;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + hf * 8);
  }
  TopList<KMAX> top;
  top.init();

  for (int j0 = 0; j0 < c_max; j0 += TNS) {
    // stage 64 span keys: 16 lanes x 16 bytes per key
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i, row = id >> 4, piece = id & 15;
      int64_t j = j0 + row;
      j = j < c_max ? j : c_max - 1;
      const bf16_t* src = Ks ? Ks + ((int64_t)kv * n + j) * HD : K + kv * kvsh + ((j + 1) * S - 1) * kvst;
      *reinterpret_cast<uint4*>(&s_k[row * KSTR + piece * 8]) = load16(src + piece * 8);
    }
    __syncthreads();
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
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = j0 + 32 * sub + 8 * (e >> 2) + 4 * hf + (e & 3);
          const float x = j < c_q ? s[e] : -INFINITY;  // causal: only complete spans below the query's own
          top.push(x, j);
        }
      }
    }
    __syncthreads();
  }

  // merge the partner lane's list (the other 16 spans of every tile)
  {
    float pv[KMAX];
    int pj[KMAX];
#pragma unroll
    for (int e = 0; e < KMAX; ++e) {
      auto a = __builtin_amdgcn_permlane32_swap(__float_as_int(top.v[e]), __float_as_int(top.v[e]), false, false);
      auto b = __builtin_amdgcn_permlane32_swap(top.j[e], top.j[e], false, false);
      // the two results are {own, partner} in an order that depends on the lane half: take
      // the one that is not this lane's own (if both are equal either will do)
      pv[e] = __int_as_float(a[0] == __float_as_int(top.v[e]) ? a[1] : a[0]);
      pj[e] = b[0] == top.j[e] ? b[1] : b[0];
    }
#pragma unroll
    for (int e = 0; e < KMAX; ++e) top.push_any(pv[e], pj[e]);
  }
  if (hf == 0 && r < Lq) {
    int32_t* oi = idx + ((int64_t)h * Lq + r) * topk;
    float* os = scores ? scores + ((int64_t)h * Lq + r) * topk : nullptr;
    // the first topk list entries are the selection; emit them in ascending index order
#pragma unroll
    for (int e = 0; e < KMAX; ++e) {
      if (e < topk) {
        int rank = 0;
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
          rank += (u < topk && (top.j[u] < top.j[e] || (top.j[u] == top.j[e] && u < e))) ? 1 : 0;
        const bool empty = top.j[e] == kEmpty;
        oi[rank] = empty ? -1 : top.j[e];
        if (os) os[rank] = empty ? -INFINITY : top.v[e];
      }
    }
  }
}

template <int KMAX>
sl_status launch(const Problem& pb, const void* Qs, const void* K, const void* Ks, int32_t* idx,
                 float* scores, hipStream_t st) {
  const int tiles_per_head = (int)((pb.Lq + TMQ - 1) / TMQ);
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  hipLaunchKernelGGL((prefill_search_mfma_kernel<KMAX>), dim3(pb.Hq * tiles_per_head), dim3(256), 0,
                     st, static_cast<const bf16_t*>(Qs), static_cast<const bf16_t*>(K),
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
