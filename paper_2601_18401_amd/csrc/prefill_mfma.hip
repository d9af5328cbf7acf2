// Prefill span-attention on the matrix cores (bf16, D = 128, S a multiple of 64).
//
// Every (head, query) row picks its own spans, so a query-stationary tile has no shared K
// operand.  Following the bucketing idea of Section 4.3 (group (query, span) pairs by the key
// blocks they touch; on the fixed span grid a bucket is simply (kv head, span)), the routed part
// makes the SPAN stationary:
//
//   bucket_count / bucket_scan / bucket_tiles / bucket_fill   invert idx into per-(kv, span)
//                                   lists of query rows (integer work, LDS histograms)
//   span_flash<false>               one workgroup per (bucket, 128-row tile): gathered Q rows
//                                   against the span's K/V tiles staged through LDS, flash
//                                   softmax, MFMA QK^T and PV; writes a normalised partial
//                                   (o, lse) per (row, slot)
//   span_flash<true>                the local window [c*S, i]: regular 128-row tiles of one
//                                   head with the causal mask; writes the row's last partial
//   merge_partials                  streaming log-sum-exp merge of the <= topk + 1 partials of
//                                   every row; writes O and LSE
//
// MFMA formulation.  Both products are computed transposed so that a lane owns a query column:
//   S^T[kv][q] = K[kv][:] . Q[q][:]      A = K tile (LDS), B = Q rows (registers)
//   O^T[d][q] += V^T[d][kv] . P^T[kv][q] A = V^T tile (LDS), B = P^T straight from the S^T
//                                         accumulators (no shuffle: the K rows of a tile are fed
//                                         in an order that makes a lane's 8 consecutive
//                                         accumulators 8 consecutive kv positions)
// With v_mfma_f32_32x32x16_bf16, lane l of the 32x32 result holds column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 for accumulator r = 0..15.
#include "kernels.h"

namespace sl {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int TM = 128;            // query rows per workgroup: 4 wavefronts x 32 columns
constexpr int TN = 64;             // kv positions per staged tile
constexpr int HD = 128;            // head dimension of this path
constexpr int KSTR = HD + 8;       // LDS row stride of the K tile, bf16 elements (272 B: conflict-free b128 reads)
constexpr int VSTR = TN + 8;       // LDS row stride of the V^T tile (144 B)
constexpr int OSTR = HD + 8;       // LDS row stride of the output staging tile
constexpr int kFlashThreads = 256;
constexpr int kBucketRows = 1024;  // query rows of one head per bucketing workgroup

struct __align__(16) FlashSmem {
  union {
    struct {
      bf16_t k[TN * KSTR];   // 17408 B
      bf16_t vt[HD * VSTR];  // 18432 B
    } kv;
    bf16_t o[TM * OSTR];     // 34816 B, epilogue only
  };
  int row_q[TM];             // element offset of the row's Q vector
  int64_t row_out[TM];       // partial index (routed) or output row index (local); -1 = no row
  float row_lse[TM];
};

__device__ __forceinline__ float pair_max(float x) {
  // lanes l and l^32 hold the two halves of a query column
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}

// ------------------------------------------------------------------ V transpose (workspace)
// Vt[kv][d][t] = V[kv][t][d], row length Lp (L rounded up to 64, zero padded).
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16_t* __restrict__ V,
                                                          bf16_t* __restrict__ Vt, int64_t L,
                                                          int64_t Lp, int64_t kvsh, int64_t kvst) {
  __shared__ bf16_t s[64 * (HD + 2)];
  const int kv = blockIdx.y, tid = threadIdx.x;
  const int64_t t0 = (int64_t)blockIdx.x * 64;
  for (int i = 0; i < 4; ++i) {
    const int idx = tid + 256 * i, row = idx >> 4, piece = idx & 15;
    const int64_t t = t0 + row;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (t < L) v = load16(V + kv * kvsh + t * kvst + piece * 8);
    uint32_t* dst = reinterpret_cast<uint32_t*>(&s[row * (HD + 2) + piece * 8]);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  __syncthreads();
  for (int i = 0; i < 4; ++i) {
    const int idx = tid + 256 * i, d = idx >> 3, piece = idx & 7;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t lo = s[(piece * 8 + 2 * e) * (HD + 2) + d];
      const uint32_t hi = s[(piece * 8 + 2 * e + 1) * (HD + 2) + d];
      w[e] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4*>(Vt + ((int64_t)kv * HD + d) * Lp + t0 + piece * 8) =
        make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// ------------------------------------------------------------------ bucketing
__global__ void zero_i32_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// grid (ceil(Lq / kBucketRows), Hq).  FILL = false: count items per (kv, span).  FILL = true:
// reserve a range per non-empty bin with one global atomic, then scatter the row ids.
template <bool FILL>
__global__ __launch_bounds__(256) void bucket_kernel(const int32_t* __restrict__ idx,
                                                     int* __restrict__ g_count,
                                                     int* __restrict__ g_cursor,
                                                     int* __restrict__ items, int64_t Lq,
                                                     int64_t q_pos0, int G, int S, int topk, int n) {
  extern __shared__ int s_hist[];  // [n] counts, then (FILL) [n] bases
  int* s_base = s_hist + n;
  const int h = blockIdx.y, kv = h / G, hl = h % G, tid = threadIdx.x;
  const int64_t r0 = (int64_t)blockIdx.x * kBucketRows;
  for (int b = tid; b < n; b += 256) s_hist[b] = 0;
  __syncthreads();
  for (int i = 0; i < kBucketRows / 256; ++i) {
    const int64_t r = r0 + tid + 256 * i;
    if (r < Lq) {
      const int64_t c = (q_pos0 + r) / S;
      const int32_t* row = idx + ((int64_t)h * Lq + r) * topk;
      for (int s = 0; s < topk; ++s) {
        const int j = row[s];
        if (j >= 0 && j < c) atomicAdd(&s_hist[j], 1);
      }
    }
  }
  __syncthreads();
  if (!FILL) {
    for (int b = tid; b < n; b += 256)
      if (s_hist[b]) atomicAdd(&g_count[kv * n + b], s_hist[b]);
    return;
  }
  for (int b = tid; b < n; b += 256) {
    const int cnt = s_hist[b];
    s_base[b] = cnt ? atomicAdd(&g_cursor[kv * n + b], cnt) : 0;
    s_hist[b] = 0;
  }
  __syncthreads();
  for (int i = 0; i < kBucketRows / 256; ++i) {
    const int64_t r = r0 + tid + 256 * i;
    if (r < Lq) {
      const int64_t c = (q_pos0 + r) / S;
      const int32_t* row = idx + ((int64_t)h * Lq + r) * topk;
      for (int s = 0; s < topk; ++s) {
        const int j = row[s];
        if (j >= 0 && j < c) items[s_base[j] + atomicAdd(&s_hist[j], 1)] = (int)(hl * Lq + r);
      }
    }
  }
}

// One workgroup: exclusive scans of the item counts and of the tile counts over the B buckets.
// item_off[B] / tile_off[B] receive the totals; cursor[b] = item_off[b] for the fill pass.
__global__ __launch_bounds__(1024) void bucket_scan_kernel(const int* __restrict__ g_count,
                                                           int* __restrict__ item_off,
                                                           int* __restrict__ tile_off,
                                                           int* __restrict__ g_cursor, int B) {
  __shared__ int s_items[1024], s_tiles[1024];
  const int tid = threadIdx.x;
  const int per = (B + 1023) / 1024;
  const int b0 = tid * per, b1 = min(B, b0 + per);
  int ni = 0, nt = 0;
  for (int b = b0; b < b1; ++b) {
    const int cnt = g_count[b];
    ni += cnt;
    nt += (cnt + TM - 1) / TM;
  }
  s_items[tid] = ni;
  s_tiles[tid] = nt;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan
    const int a = tid >= off ? s_items[tid - off] : 0;
    const int t = tid >= off ? s_tiles[tid - off] : 0;
    __syncthreads();
    s_items[tid] += a;
    s_tiles[tid] += t;
    __syncthreads();
  }
  int io = s_items[tid] - ni, to = s_tiles[tid] - nt;
  for (int b = b0; b < b1; ++b) {
    const int cnt = g_count[b];
    item_off[b] = io;
    tile_off[b] = to;
    g_cursor[b] = io;
    io += cnt;
    to += (cnt + TM - 1) / TM;
  }
  if (tid == 1023) {
    item_off[B] = s_items[1023];
    tile_off[B] = s_tiles[1023];
  }
}

// One workgroup per bucket writes the bucket id of each of its tiles.
__global__ __launch_bounds__(256) void bucket_tiles_kernel(const int* __restrict__ tile_off,
                                                           int* __restrict__ tile_bucket) {
  const int b = blockIdx.x;
  const int t0 = tile_off[b], t1 = tile_off[b + 1];
  for (int t = t0 + threadIdx.x; t < t1; t += 256) tile_bucket[t] = b;
}

// ------------------------------------------------------------------ flash tile
struct FlashArgs {
  const bf16_t* Q;
  const bf16_t* K;
  const bf16_t* Vt;
  const int32_t* idx;
  // routed
  const int* item_off;
  const int* tile_off;
  const int* tile_bucket;
  const int* items;
  bf16_t* part_o;
  float* part_lse;
  // local + merge
  bf16_t* O;
  float* LSE;
  int64_t L, Lp, Lq, q_pos0;
  int Hq, G, S, topk, n;
  float scale_log2e;
  int64_t qsh, qst, kvsh, kvst;
};

__device__ __forceinline__ int perm_row(int rho) {
  // swap bits 2 and 3: accumulator order <-> consecutive kv positions
  return (rho & 0x13) | ((rho & 4) << 1) | ((rho & 8) >> 1);
}

template <bool LOCAL>
__global__ __launch_bounds__(kFlashThreads, 2) void span_flash_kernel(const FlashArgs a) {
  __shared__ FlashSmem sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qc = lane & 31, hf = lane >> 5;
  const int qrow = wave * 32 + qc;

  int kv;
  int64_t kv_begin, kv_end;  // staged kv range [kv_begin, kv_end), multiple of TN long
  int h_local = 0;
  int64_t r0 = 0;
  if (!LOCAL) {
    // XCD-aware block -> tile map: blocks b, b+8, b+16, ... run on one XCD and take consecutive
    // tiles, so the tiles of a bucket share that XCD's L2 copy of the span.
    const int T = a.tile_off[a.Hq / a.G * a.n];
    const int per = (T + 7) / 8;
    const int bx = blockIdx.x;
    if (bx / 8 >= per) return;
    const int t = (bx % 8) * per + bx / 8;
    if (t >= T) return;
    const int b = a.tile_bucket[t];
    kv = b / a.n;
    const int j = b % a.n;
    const int i0 = a.item_off[b] + (t - a.tile_off[b]) * TM;
    const int i1 = a.item_off[b + 1];
    if (tid < TM) {
      const int it = i0 + tid;
      int64_t out = -1;
      int qoff = 0;
      const int id = a.items[it < i1 ? it : i1 - 1];
      const int hl = id / (int)a.Lq;
      const int64_t r = id - (int64_t)hl * a.Lq;
      const int h = kv * a.G + hl;
      qoff = (int)(h * a.qsh + r * a.qst);
      if (it < i1) {
        const int32_t* row = a.idx + ((int64_t)h * a.Lq + r) * a.topk;
        for (int s = a.topk - 1; s >= 0; --s)  // first slot that lists the span
          if (row[s] == j) out = ((int64_t)h * a.Lq + r) * (a.topk + 1) + s;
      }
      sm.row_q[tid] = qoff;
      sm.row_out[tid] = out;
    }
    kv_begin = (int64_t)j * a.S;
    kv_end = kv_begin + a.S;
  } else {
    const int tiles_per_head = (int)((a.Lq + TM - 1) / TM);
    const int h = blockIdx.x / tiles_per_head;
    r0 = (int64_t)(blockIdx.x % tiles_per_head) * TM;
    kv = h / a.G;
    h_local = h;
    if (tid < TM) {
      const int64_t r = r0 + tid;
      const int64_t rc = r < a.Lq ? r : a.Lq - 1;
      sm.row_q[tid] = (int)(h * a.qsh + rc * a.qst);
      sm.row_out[tid] = r < a.Lq ? ((int64_t)h * a.Lq + r) * (a.topk + 1) + a.topk : -1;
    }
    const int64_t i_first = a.q_pos0 + r0;
    const int64_t i_last = min(a.q_pos0 + r0 + TM - 1, a.q_pos0 + a.Lq - 1);
    kv_begin = (i_first / a.S) * a.S;
    kv_end = kv_begin + ((i_last - kv_begin) / TN + 1) * TN;
  }
  __syncthreads();

  // Q rows of this lane's column, as the B operand of S^T = K Q^T
  bf16x8 qf[8];
  {
    const bf16_t* qp = a.Q + sm.row_q[qrow];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + hf * 8);
  }
  int64_t i_q = 0, lo_q = 0;
  if (LOCAL) {
    i_q = a.q_pos0 + min(r0 + qrow, a.Lq - 1);
    lo_q = (i_q / a.S) * a.S;
  }

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const bf16_t* Kb = a.K + (int64_t)kv * a.kvsh;
  const bf16_t* Vtb = a.Vt + (int64_t)kv * HD * a.Lp;
  const int krow = perm_row(qc);

  for (int64_t t0 = kv_begin; t0 < kv_end; t0 += TN) {
    // stage K [TN][HD] and V^T [HD][TN]
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + kFlashThreads * i, row = id >> 4, piece = id & 15;
      int64_t tok = t0 + row;
      if (LOCAL) tok = tok < a.L ? tok : a.L - 1;
      const uint4 v = load16(Kb + tok * a.kvst + piece * 8);
      *reinterpret_cast<uint4*>(&sm.kv.k[row * KSTR + piece * 8]) = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + kFlashThreads * i, d = id >> 3, piece = id & 7;
      const uint4 v = load16(Vtb + (int64_t)d * a.Lp + t0 + piece * 8);
      *reinterpret_cast<uint4*>(&sm.kv.vt[d * VSTR + piece * 8]) = v;
    }
    __syncthreads();

    // S^T = K Q^T for the two 32-row halves of the tile
    f32x16 s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 ka =
            *reinterpret_cast<const bf16x8*>(&sm.kv.k[(32 * sub + krow) * KSTR + kk * 16 + hf * 8]);
        s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[kk], s[sub], 0, 0, 0);
      }
    }

    // logits in log2 units, mask (local window only), running max
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = s[sub][r] * a.scale_log2e;
        if (LOCAL) {
          const int64_t t = t0 + 32 * sub + 16 * (r >> 3) + 8 * hf + (r & 7);
          x = (t <= i_q && t >= lo_q) ? x : -INFINITY;
        }
        s[sub][r] = x;
        mx = fmaxf(mx, x);
      }
    mx = pair_max(mx);
    const float m_new = fmaxf(m, mx);
    const float m_use = m_new > -INFINITY ? m_new : 0.f;  // whole column masked so far
    const float alpha = fast_exp2(m - m_use);
    m = m_new;
    l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;

    bf16x8 pb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      f32x8 p;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = fast_exp2(s[ks >> 1][8 * (ks & 1) + e] - m_use);
        l += p[e];
      }
      pb[ks] = __builtin_convertvector(p, bf16x8);
    }

    // O^T += V^T P^T
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const bf16x8 va =
            *reinterpret_cast<const bf16x8*>(&sm.kv.vt[(32 * dt + qc) * VSTR + ks * 16 + hf * 8]);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[ks], o[dt], 0, 0, 0);
      }
    __syncthreads();
  }

  // epilogue: normalise, stage the tile as [row][d] bf16 in LDS
  const float lt = pair_sum(l);
  const float inv = 1.f / lt;
  if (hf == 0) sm.row_lse[qrow] = (m + __log2f(lt)) * kLn2;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int d = 32 * dt + 8 * g4 + 4 * hf;
      uint32_t w0 = (uint32_t)f32_to_bf16(o[dt][4 * g4 + 0] * inv) |
                    ((uint32_t)f32_to_bf16(o[dt][4 * g4 + 1] * inv) << 16);
      uint32_t w1 = (uint32_t)f32_to_bf16(o[dt][4 * g4 + 2] * inv) |
                    ((uint32_t)f32_to_bf16(o[dt][4 * g4 + 3] * inv) << 16);
      *reinterpret_cast<uint2*>(&sm.o[qrow * OSTR + d]) = make_uint2(w0, w1);
    }
  __syncthreads();

  // 16 lanes per row, 16 bytes per lane
  for (int pass = 0; pass < TM / 16; ++pass) {
    const int row = pass * 16 + (tid >> 4), piece = tid & 15;
    const int64_t out = sm.row_out[row];
    if (out < 0) continue;
    const uint4 mine = *reinterpret_cast<const uint4*>(&sm.o[row * OSTR + piece * 8]);
    *reinterpret_cast<uint4*>(a.part_o + out * HD + piece * 8) = mine;
    if (piece == 0) a.part_lse[out] = sm.row_lse[row];
  }
}

// ------------------------------------------------------------------ merge
// Log-sum-exp merge of a row's partials: up to topk routed slots plus the local window (slot
// topk).  16 lanes per row, 16 bytes per lane; every load of a lane is issued before the first
// dependent use, so the kernel streams at HBM rate.
template <int KMAX>
__global__ __launch_bounds__(256) void merge_partials_kernel(
    const int32_t* __restrict__ idx, const bf16_t* __restrict__ part_o,
    const float* __restrict__ part_lse, bf16_t* __restrict__ O, float* __restrict__ LSE,
    int64_t rows, int64_t Lq, int64_t q_pos0, int S, int topk) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int piece = threadIdx.x & 15;
  if (row >= rows) return;
  const int64_t r = row % Lq;
  const int c = (int)((q_pos0 + r) / S);
  const int nslot = topk + 1;
  const int32_t* irow = idx + row * topk;
  const float* lrow = part_lse + row * nslot;
  const bf16_t* orow = part_o + row * nslot * HD + piece * 8;

  int js[KMAX];
  float ls[KMAX + 1];
  uint4 ov[KMAX + 1];
#pragma unroll
  for (int s = 0; s < KMAX; ++s) js[s] = s < topk ? irow[s] : -1;
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    // a slot takes part if its span is a candidate and no earlier slot lists the same span
    bool ok = js[s] >= 0 && js[s] < c;
#pragma unroll
    for (int u = 0; u < s; ++u) ok = ok && js[u] != js[s];
    ls[s] = ok ? lrow[s] : -INFINITY;
    ov[s] = ok ? load16(orow + (int64_t)s * HD) : make_uint4(0, 0, 0, 0);
  }
  ls[KMAX] = lrow[topk];
  ov[KMAX] = load16(orow + (int64_t)topk * HD);

  float M = ls[KMAX];
#pragma unroll
  for (int s = 0; s < KMAX; ++s) M = fmaxf(M, ls[s]);
  float acc[8], f[8];
  float wsum = __expf(ls[KMAX] - M);
  Elem<bf16_t>::unpack(ov[KMAX], f);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = wsum * f[e];
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    const float w = ls[s] > -INFINITY ? __expf(ls[s] - M) : 0.f;
    wsum += w;
    Elem<bf16_t>::unpack(ov[s], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, f[e], acc[e]);
  }
  const float winv = 1.f / wsum;
  uint4 res;
  res.x = (uint32_t)f32_to_bf16(acc[0] * winv) | ((uint32_t)f32_to_bf16(acc[1] * winv) << 16);
  res.y = (uint32_t)f32_to_bf16(acc[2] * winv) | ((uint32_t)f32_to_bf16(acc[3] * winv) << 16);
  res.z = (uint32_t)f32_to_bf16(acc[4] * winv) | ((uint32_t)f32_to_bf16(acc[5] * winv) << 16);
  res.w = (uint32_t)f32_to_bf16(acc[6] * winv) | ((uint32_t)f32_to_bf16(acc[7] * winv) << 16);
  *reinterpret_cast<uint4*>(O + row * HD + piece * 8) = res;
  if (piece == 0) LSE[row] = M + __logf(wsum);
}

// ------------------------------------------------------------------ workspace carving
struct MfmaWs {
  size_t vt, counts, item_off, tile_off, cursor, tile_bucket, items, part_lse, part_o, total;
  int64_t Lp;
  int B, max_tiles;
  int64_t max_items;
};

MfmaWs carve(const Problem& pb) {
  MfmaWs w;
  w.Lp = (int64_t)align_up((size_t)pb.L, 64);
  w.B = pb.Hkv * (int)pb.n;
  w.max_items = (int64_t)pb.Hq * pb.Lq * pb.topk;
  w.max_tiles = (int)((w.max_items + TM - 1) / TM) + w.B;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  w.vt = take((size_t)pb.Hkv * HD * w.Lp * sizeof(bf16_t));
  w.counts = take((size_t)w.B * sizeof(int));
  w.item_off = take((size_t)(w.B + 1) * sizeof(int));
  w.tile_off = take((size_t)(w.B + 1) * sizeof(int));
  w.cursor = take((size_t)w.B * sizeof(int));
  w.tile_bucket = take((size_t)w.max_tiles * sizeof(int));
  w.items = take((size_t)w.max_items * sizeof(int));
  const size_t nparts = (size_t)pb.Hq * pb.Lq * (pb.topk + 1);  // routed slots + the local window
  w.part_lse = take(nparts * sizeof(float));
  w.part_o = take(nparts * HD * sizeof(bf16_t));
  w.total = off;
  return w;
}

}  // namespace

bool prefill_attention_mfma_supported(const Problem& pb) {
  return pb.dtype == SL_BF16 && pb.D == HD && pb.S % TN == 0 && pb.n <= 4096 &&
         (int64_t)pb.G * pb.Lq < ((int64_t)1 << 31) &&
         (int64_t)pb.Hq * pb.Lq * (pb.topk + 1) < ((int64_t)1 << 31) &&
         // row_q holds 32-bit element offsets into Q
         (int64_t)pb.Hq * pb.qsh + pb.Lq * pb.qst < ((int64_t)1 << 31);
}

size_t prefill_attention_mfma_ws_bytes(const Problem& pb) { return carve(pb).total; }

sl_status prefill_attention_mfma(const Problem& pb, const void* Q, const void* K, const void* V,
                                 const int32_t* idx, void* O, float* LSE, void* ws,
                                 hipStream_t st) {
  const MfmaWs w = carve(pb);
  char* base = static_cast<char*>(ws);
  bf16_t* Vt = reinterpret_cast<bf16_t*>(base + w.vt);
  int* counts = reinterpret_cast<int*>(base + w.counts);
  int* item_off = reinterpret_cast<int*>(base + w.item_off);
  int* tile_off = reinterpret_cast<int*>(base + w.tile_off);
  int* cursor = reinterpret_cast<int*>(base + w.cursor);
  int* tile_bucket = reinterpret_cast<int*>(base + w.tile_bucket);
  int* items = reinterpret_cast<int*>(base + w.items);
  float* part_lse = reinterpret_cast<float*>(base + w.part_lse);
  bf16_t* part_o = reinterpret_cast<bf16_t*>(base + w.part_o);
  const int n = (int)pb.n;

  hipLaunchKernelGGL(transpose_v_kernel, dim3((unsigned)(w.Lp / 64), pb.Hkv), dim3(256), 0, st,
                     static_cast<const bf16_t*>(V), Vt, pb.L, w.Lp, pb.kvsh, pb.kvst);

  FlashArgs a;
  a.Q = static_cast<const bf16_t*>(Q);
  a.K = static_cast<const bf16_t*>(K);
  a.Vt = Vt;
  a.idx = idx;
  a.item_off = item_off;
  a.tile_off = tile_off;
  a.tile_bucket = tile_bucket;
  a.items = items;
  a.part_o = part_o;
  a.part_lse = part_lse;
  a.O = static_cast<bf16_t*>(O);
  a.LSE = LSE;
  a.L = pb.L;
  a.Lp = w.Lp;
  a.Lq = pb.Lq;
  a.q_pos0 = pb.q_pos0;
  a.Hq = pb.Hq;
  a.G = pb.G;
  a.S = pb.S;
  a.topk = pb.topk;
  a.n = n;
  a.scale_log2e = pb.scale * kLog2e;
  a.qsh = pb.qsh;
  a.qst = pb.qst;
  a.kvsh = pb.kvsh;
  a.kvst = pb.kvst;

  if (pb.topk > 0) {
    const dim3 bgrid((unsigned)((pb.Lq + kBucketRows - 1) / kBucketRows), pb.Hq);
    hipLaunchKernelGGL(zero_i32_kernel, dim3((w.B + 255) / 256), dim3(256), 0, st, counts, w.B);
    hipLaunchKernelGGL(bucket_kernel<false>, bgrid, dim3(256), (size_t)n * sizeof(int), st, idx,
                       counts, cursor, items, pb.Lq, pb.q_pos0, pb.G, pb.S, pb.topk, n);
    hipLaunchKernelGGL(bucket_scan_kernel, dim3(1), dim3(1024), 0, st, counts, item_off, tile_off,
                       cursor, w.B);
    hipLaunchKernelGGL(bucket_tiles_kernel, dim3(w.B), dim3(256), 0, st, tile_off, tile_bucket);
    hipLaunchKernelGGL(bucket_kernel<true>, bgrid, dim3(256), (size_t)2 * n * sizeof(int), st, idx,
                       counts, cursor, items, pb.Lq, pb.q_pos0, pb.G, pb.S, pb.topk, n);
    if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
    const int grid = (int)align_up((size_t)w.max_tiles, 8);
    if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
    hipLaunchKernelGGL(span_flash_kernel<false>, dim3(grid), dim3(kFlashThreads), 0, st, a);
    if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  }
  const int tiles_per_head = (int)((pb.Lq + TM - 1) / TM);
  hipLaunchKernelGGL(span_flash_kernel<true>, dim3(pb.Hq * tiles_per_head), dim3(kFlashThreads), 0,
                     st, a);
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  const dim3 mgrid((unsigned)((rows + 15) / 16));
#define SL_MERGE(KM)                                                                             \
  hipLaunchKernelGGL(merge_partials_kernel<KM>, mgrid, dim3(256), 0, st, idx, part_o, part_lse,  \
                     a.O, LSE, rows, pb.Lq, pb.q_pos0, pb.S, pb.topk)
  if (pb.topk == 0) SL_MERGE(1);
  else if (pb.topk <= 8) SL_MERGE(8);
  else if (pb.topk <= 16) SL_MERGE(16);
  else SL_MERGE(32);
#undef SL_MERGE
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

}  // namespace sl
