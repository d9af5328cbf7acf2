// Prefill span-attention on the matrix cores (bf16, D = 128, S a multiple of 64).
//
// Every (head, query) row picks its own spans, so a query-stationary tile has no shared K
// operand.  Following the bucketing idea of Section 4.3 (group (query, span) pairs by the key
// blocks they touch; on the fixed span grid a bucket is simply (kv head, span)), the routed part
// makes the SPAN stationary:
//
//   bucket_count / bucket_scan / bucket_tiles / bucket_fill   invert idx into per-(kv, span)
//                                   lists of query rows (integer work, LDS histograms)
//   span_flash_routed               persistent workgroups walk the (bucket, 256-row tile) list:
//                                   gathered Q rows against the span's K/V tiles staged through
//                                   LDS, flash softmax, MFMA QK^T and PV; writes a normalised
//                                   partial (o, lse) per (row, slot)
//   span_flash_local                the local window [c*S, i]: regular 128-row tiles of one
//                                   head with the causal mask; joint form with topk <= 8: merges
//                                   the row's routed partials in its epilogue (log-sum-exp) and
//                                   writes O and LSE; otherwise writes the row's last partial
//   merge_partials / merge_combined streaming merge of the <= topk + 1 partials of every row
//                                   (topk > 8, and the gated combination of Section 3.4)
//
// MFMA formulation.  Both products are computed transposed so that a lane owns a query column:
//   S^T[kv][q] = K[kv][:] . Q[q][:]      A = K tile (LDS), B = Q rows (registers)
//   O^T[d][q] += V^T[d][kv] . P^T[kv][q] A = V^T tile (LDS), B = P^T straight from the S^T
//                                         accumulators (no shuffle: the K rows of a tile are fed
//                                         in an order that makes a lane's 8 consecutive
//                                         accumulators 8 consecutive kv positions)
// With v_mfma_f32_32x32x16_bf16, lane l of the 32x32 result holds column l%32 and rows
// 8*(r/4) + 4*(l/32) + r%4 for accumulator r = 0..15.
#include <mutex>

#include "kernels.h"

namespace sl {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int TG = 128;            // rows of one wavefront group (4 wavefronts x 32 columns)
constexpr int TN = 64;             // kv positions per staged tile
constexpr int HD = 128;            // head dimension of this path
constexpr int kBucketRows = 4096;  // query rows of one head per bucketing workgroup

// LDS of the flash kernels (dynamic).  Main loop: stages of the V^T tile and of the K tile, filled
// by direct global->LDS loads (16 bytes per lane, a wavefront instruction fills 1 KB
// contiguously); rows are unpadded and their 16-byte pieces XOR-swizzled so that the MFMA
// operand reads of 16 consecutive lanes hit 16 distinct bank groups:
//   K tile  [64][128]: piece p of row r at position p ^ (r & 15)
//   V^T tile [128][64]: piece p of row d at position p ^ ((d >> 1) & 7)
// Epilogue: each wavefront group stages its output tile [128][128] bf16 (piece p of row r at
// p ^ (r & 15)).
//   NG = 2 (routed, 512 threads, 256 rows, one workgroup per compute unit, 154624 bytes): two K
//     and three V^T stages (the late group reads a V^T tile one step after the early group); the
//     output region is separate, so the first K/V tile of the next 256-row tile can be fetched
//     while the current one is written out.
//   NG = 1 (local window, 256 threads, 128 rows, 67072 bytes: two workgroups per compute unit, so
//     one's epilogue runs beside the other's main loop): two stages each; the output region
//     lies over the V^T stages, which are dead by then.
constexpr int kStageElems = TN * HD;  // 8192 bf16 = 16 KB
template <int NG>
struct FlashLds {
  static constexpr int kStagesK = 2, kStagesV = NG == 2 ? 3 : 2;
  static constexpr int kV = 0;
  static constexpr int kK = kStagesV * kStageElems * 2;
  static constexpr int kStagesEnd = (kStagesV + kStagesK) * kStageElems * 2;
  static constexpr int kOut = NG == 2 ? kStagesEnd : 0;                             // bf16[NG][TG][HD]
  static constexpr int kRowOut = NG == 2 ? kOut + NG * TG * HD * 2 : kStagesEnd;    // int64[NG][TG]
  static constexpr int kRowLse = kRowOut + NG * TG * 8;                             // float[NG][TG]
  // NG = 2: per wavefront 256 bytes for the next tile's record and 256 for its items, fetched by
  // direct global->LDS loads while the current tile runs (they hold no registers meanwhile)
  static constexpr int kAhead = kRowLse + NG * TG * 4;
  static constexpr int kBytes = kAhead + (NG == 2 ? 8 * 512 : 0);
  static constexpr int kThreads = NG * 256;
  static constexpr int kRows = NG * TG;  // query rows per workgroup
  static constexpr int kBlocksPerWave = 16 / (4 * NG);  // 1 KB blocks of a staged tile per wavefront
};
constexpr int TM = FlashLds<2>::kRows;  // rows of a routed tile

#define SL_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define SL_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ float pair_max(float x) {
  // lanes l and l^32 hold the two halves of a query column
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}

// The paper's geometry: token range [lo, hi) that slot anchor t contributes for the query at i
// (S_t minus the window, Algorithm 1's DedupConcat(S_t, W) being that range followed by W).
// ell = l(i).  valid: t is an anchor of this query at all; the range may still be empty.
struct AnchorSpan {
  int64_t lo, hi;
  bool valid;
};
__device__ __forceinline__ AnchorSpan anchor_span_of(int64_t i, int64_t t, int64_t ell, int64_t window, int ab,
                                                     int af) {
  AnchorSpan r;
  r.valid = t >= 0 && t <= i;
  const int64_t wlo = window > 0 ? (i - window + 1 > 0 ? i - window + 1 : 0) : i + 1;
  r.lo = t - ab * ell > 0 ? t - ab * ell : 0;
  const int64_t e1 = t + af * ell < i ? t + af * ell : i;
  r.hi = (e1 < wlo - 1 ? e1 : wlo - 1) + 1;
  if (r.hi < r.lo || !r.valid) r.hi = r.lo;
  return r;
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
// Inverts idx into per-(kv head, span) lists of (row, slot) items without a sort and without
// global atomics, so that the item order is the same on every run: within a bucket the items come
// by query head of the group, then by query row.
//   bucket_kernel<false>      grid (chunks of kBucketRows rows, Hq): LDS histogram of the block's
//                             items per span -> blk_cnt[h][chunk][span]
//   bucket_block_scan_kernel  per (kv head, span): exclusive scan of blk_cnt over (head of the
//                             group, chunk), in place; the total goes to g_count
//   bucket_scan_kernel / bucket_tiles_kernel   bucket offsets and tile records
//   bucket_kernel<true>       recounts per wavefront (each owns a contiguous quarter of the block's
//                             rows), turns the counts into bases behind the block's prefix and
//                             scatters the items
template <bool FILL>
__global__ __launch_bounds__(256) void bucket_kernel(const int32_t* __restrict__ idx,
                                                     int* __restrict__ blk_cnt,
                                                     const int* __restrict__ g_cursor,
                                                     int* __restrict__ items, int64_t Lq,
                                                     int64_t q_pos0, int G, int S, int topk, int n) {
  extern __shared__ int s_hist[];  // count pass: [n]; fill pass: [4][n], one histogram per wavefront
  const int h = blockIdx.y, kv = h / G, hl = h % G;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int64_t r0 = (int64_t)blockIdx.x * kBucketRows + wave * (kBucketRows / 4);
  int* const blk = blk_cnt + ((int64_t)h * gridDim.x + blockIdx.x) * n;
  int* const hist = FILL ? s_hist + wave * n : s_hist;
  for (int b = tid; b < (FILL ? 4 : 1) * n; b += 256) s_hist[b] = 0;
  __syncthreads();
  auto for_items = [&](auto f) {
    for (int i = 0; i < kBucketRows / 256; ++i) {
      const int64_t r = r0 + 64 * i + lane;
      if (r < Lq) {
        const int64_t c = (q_pos0 + r) / S;
        const int32_t* row = idx + ((int64_t)h * Lq + r) * topk;
        for (int s = 0; s < topk; ++s) {
          const int j = row[s];
          if (j >= 0 && j < c) f(j, r, s);
        }
      }
    }
  };
  for_items([&](int j, int64_t, int) { atomicAdd(&hist[j], 1); });
  __syncthreads();
  if (!FILL) {
    for (int b = tid; b < n; b += 256) blk[b] = s_hist[b];
    return;
  }
  for (int b = tid; b < n; b += 256) {
    int base = g_cursor[kv * n + b] + blk[b];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int cnt = s_hist[w * n + b];
      s_hist[w * n + b] = base;
      base += cnt;
    }
  }
  __syncthreads();
  for_items([&](int j, int64_t r, int s) { items[atomicAdd(&hist[j], 1)] = (int)(((hl * Lq + r) << 5) | s); });
}

// grid (ceil(n / 32), Hkv), 256 threads = 32 spans x 8 segments of the E = G * chunks block counts
// of a (kv head, span): exclusive scan in place, total to g_count.
__global__ __launch_bounds__(256) void bucket_block_scan_kernel(int* __restrict__ blk_cnt,
                                                                int* __restrict__ g_count, int E, int n) {
  __shared__ int s_tot[8][32];
  const int bl = threadIdx.x & 31, seg = threadIdx.x >> 5;
  const int b = blockIdx.x * 32 + bl, kv = blockIdx.y;
  const int per = (E + 7) / 8, e0 = seg * per, e1 = min(E, e0 + per);
  int* const col = blk_cnt + (int64_t)kv * E * n + b;
  int sum = 0;
  if (b < n) {
    for (int e = e0; e < e1; e += 8) {
      int v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = e + u < e1 ? col[(int64_t)(e + u) * n] : 0;
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += v[u];
    }
  }
  s_tot[seg][bl] = sum;
  __syncthreads();
  if (b >= n) return;
  int run = 0;
  for (int s2 = 0; s2 < seg; ++s2) run += s_tot[s2][bl];
  for (int e = e0; e < e1; e += 8) {
    int v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = e + u < e1 ? col[(int64_t)(e + u) * n] : 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (e + u < e1) col[(int64_t)(e + u) * n] = run;
      run += v[u];
    }
  }
  if (seg == 7) g_count[kv * n + b] = run;
}

// The same two passes for the paper's geometry: an item is a (row, slot) whose anchor is valid and
// whose span minus the window is not empty; its bucket is (kv head, block of E tokens that holds the
// span's last token).  Blocks of one kv head are ordered by (chunk of rows, head of the group), so
// that a bucket's items come by query position first: the rows of a tile then have nearly the
// same span length.  The fill pass also marks the partial of a valid anchor with an empty span
// as empty (lse = -inf) for the merge.
template <bool FILL>
__global__ __launch_bounds__(256) void bucket_anchor_kernel(const int32_t* __restrict__ anchors,
                                                            int* __restrict__ blk_cnt,
                                                            const int* __restrict__ g_cursor,
                                                            int* __restrict__ items,
                                                            float* __restrict__ part_lse, int64_t Lq,
                                                            int64_t q_pos0, int G, int topk, int n,
                                                            int64_t window, int ab, int af, int aroot, int E) {
  extern __shared__ int s_hist[];  // count pass: [n]; fill pass: [4][n], one histogram per wavefront
  const int h = blockIdx.y, kv = h / G, hl = h % G;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int64_t r0 = (int64_t)blockIdx.x * kBucketRows + wave * (kBucketRows / 4);
  int* const blk = blk_cnt + (((int64_t)kv * gridDim.x + blockIdx.x) * G + hl) * n;
  int* const hist = FILL ? s_hist + wave * n : s_hist;
  for (int b = tid; b < (FILL ? 4 : 1) * n; b += 256) s_hist[b] = 0;
  __syncthreads();
  auto for_items = [&](auto f) {
    for (int it = 0; it < kBucketRows / 256; ++it) {
      const int64_t r = r0 + 64 * it + lane;
      if (r < Lq) {
        const int64_t i = q_pos0 + r;
        const int64_t ell = span_base_length(i, aroot);
        const int32_t* row = anchors + ((int64_t)h * Lq + r) * topk;
        for (int s = 0; s < topk; ++s) {
          const AnchorSpan sp = anchor_span_of(i, row[s], ell, window, ab, af);
          if (sp.hi > sp.lo) f((int)((sp.hi - 1) / E), r, s);
          else if (FILL && sp.valid) part_lse[((int64_t)h * Lq + r) * (topk + 1) + s] = -INFINITY;
        }
      }
    }
  };
  for_items([&](int j, int64_t, int) { atomicAdd(&hist[j], 1); });
  __syncthreads();
  if (!FILL) {
    for (int b = tid; b < n; b += 256) blk[b] = s_hist[b];
    return;
  }
  for (int b = tid; b < n; b += 256) {
    int base = g_cursor[kv * n + b] + blk[b];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int cnt = s_hist[w * n + b];
      s_hist[w * n + b] = base;
      base += cnt;
    }
  }
  __syncthreads();
  for_items([&](int j, int64_t r, int s) { items[atomicAdd(&hist[j], 1)] = (int)(((hl * Lq + r) << 5) | s); });
}

// One workgroup: exclusive scans of the item counts and of the tile counts over the B buckets.
// item_off[B] / tile_off[B] receive the totals.  The item list is laid out tile by tile, TM
// entries per tile (a bucket's last tile is padded), so that the items of tile t start at t*TM
// whatever its record says: cursor[b] = tile_off[b] * TM for the fill pass.
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
    g_cursor[b] = to * TM;
    io += cnt;
    to += (cnt + TM - 1) / TM;
  }
  if (tid == 1023) {
    item_off[B] = s_items[1023];
    tile_off[B] = s_tiles[1023];
  }
}

// One workgroup per bucket writes the record of each of its tiles,
// {bucket, first item = t*TM, number of items (1..TM), unused}, and fills the padding of the
// bucket's last tile with item 0 (row 0, slot 0 of the kv head's first query head: a valid row to
// read, whose result the flash kernel drops because the lane lies beyond the tile's item count).
__global__ __launch_bounds__(256) void bucket_tiles_kernel(const int* __restrict__ tile_off,
                                                           const int* __restrict__ item_off,
                                                           int4* __restrict__ tile_info,
                                                           int* __restrict__ items) {
  const int b = blockIdx.x;
  const int t0 = tile_off[b], t1 = tile_off[b + 1];
  const int cnt = item_off[b + 1] - item_off[b];
  for (int t = t0 + threadIdx.x; t < t1; t += 256)
    tile_info[t] = make_int4(b, t * TM, min(TM, cnt - (t - t0) * TM), 0);
  if (t1 > t0) {
    const int last = cnt - (t1 - 1 - t0) * TM;  // items of the last tile, 1..TM
    for (int e = last + threadIdx.x; e < TM; e += 256) items[(int64_t)(t1 - 1) * TM + e] = 0;
  }
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
  const int4* tile_info;
  const int* items;
  bf16_t* part_o;
  float* part_lse;
  // local + merge
  bf16_t* O;
  float* LSE;
  int64_t L, Lp, Lq, q_pos0;
  int Hq, G, S, A, topk, n;  // A: anchor spacing (= S on the disjoint grid); n = ceil(L / A)
  // The paper's own geometry (Section 3.3, Algorithm 1) instead of the grid: idx holds anchor
  // TOKENS; window > 0 marks this mode.  Span of anchor t for the query at i:
  // [max(0, t - ab*l(i)), min(i, t + af*l(i))] minus the window [i - window + 1, i], l = ceil(i^(1-1/aroot)).
  // Buckets are (kv head, end block): block e holds the spans whose last token lies in
  // [e*E, (e+1)*E), E a multiple of 64 (the key-block bucketing of Section 4.3); n = ceil(L / E).
  int64_t window;
  int ab, af, aroot, E;
  float scale_log2e;
  int64_t qsh, qst, kvsh, kvst;
};

__device__ __forceinline__ int perm_row(int rho) {
  // swap bits 2 and 3: accumulator order <-> consecutive kv positions
  return (rho & 0x13) | ((rho & 4) << 1) | ((rho & 8) >> 1);
}

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// One 256-row tile as seen by a lane: the kv head and kv range [kv_begin, kv_end) (a multiple of
// TN long) shared by the workgroup, and the lane's own query column.
struct TileDesc {
  int kv;
  int64_t kv_begin, kv_end;
  int64_t q_off;      // element offset of the lane's Q vector
  int64_t row_out;    // partial record index of the lane's column (fused merge: its row index
                      // h*Lq + r), -1 = no row
  int64_t row_base;   // fused merge: h*Lq of the tile's head
  int64_t i_q, lo_q;  // LOCAL: query position and start of its window
};

// State a workgroup carries from one tile to the next: the rotating stage indices, whether the
// tile's first K/V stage and Q fragments were already fetched by the previous tile's tail, and
// the Q fragments themselves.
struct FlashCarry {
  int kb, vb;
  bool primed;
  bool pending;  // the previous tile's output still sits in LDS (routed tiles write it out a step later)
  bf16x8 qf[8];
};

// Writes a wavefront's staged output rows (normalised partial o as bf16, lse) of a routed tile
// from the group's LDS region to the partial buffers: 16 lanes per row, 16 bytes per lane.
// Called when no direct global->LDS load is in flight (the compiler orders an LDS read after all
// outstanding vector-memory operations once such loads exist).
__device__ __forceinline__ void flush_routed_output(const FlashArgs& a, char* lds, int grp, int w4, int lane) {
  using Lds = FlashLds<2>;
  const bf16_t* const ost = reinterpret_cast<const bf16_t*>(lds + Lds::kOut) + grp * TG * HD;
  const int64_t* const row_out = reinterpret_cast<const int64_t*>(lds + Lds::kRowOut) + grp * TG;
  const float* const row_lse = reinterpret_cast<const float*>(lds + Lds::kRowLse) + grp * TG;
  const int piece = lane & 15;
  // two rows per lane at a time: the tile's accumulators are live here, registers are scarce
#pragma unroll
  for (int ub = 0; ub < 8; ub += 2) {
    int64_t outs[2];
    uint4 vals[2];
    float lses[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = w4 * 32 + (ub + u) * 4 + (lane >> 4);
      outs[u] = row_out[row];
      lses[u] = row_lse[row];
      vals[u] = *reinterpret_cast<const uint4*>(&ost[row * HD + ((piece ^ (row & 15)) << 3)]);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (outs[u] >= 0) {
        // streamed past the caches: the partials (gigabytes) are read back by a later kernel, and
        // the K/V tiles keep the L2
        store16_stream(a.part_o + outs[u] * HD + piece * 8, vals[u]);
        if (piece == 0) __builtin_nontemporal_store(lses[u], &a.part_lse[outs[u]]);
      }
    }
  }
}

// One tile of NG*128 rows.  All threads call.  If has_next, request_next() issues the caller's
// loads for the tile this workgroup processes afterwards and describe_next() turns them into
// `next`: the first is called right after the first kv step's barrier (next to that step's K/V
// loads, so the wait before the second step covers it), the second after the kv loop.
//
// The eight wavefronts form two groups of four (each group owns 128 rows, a wavefront 32
// columns); SIMD s hosts wavefront s of both groups.  Both groups consume the same staged K/V
// tiles, but the late group runs its PV product one kv tile behind:
//     early, per kv tile i:   QK(i)    softmax(i)  PV(i)
//     late,  per kv tile i:   PV(i-1)  QK(i)       softmax(i)          (+ PV(last) after the loop)
// so that between two barriers the softmax arithmetic of one group runs in the shadow of the
// other group's MFMAs instead of both groups asking for the matrix pipe at the same time.
// When the kv loop is over, the first K/V stage and the Q fragments of the next tile are
// requested before the output tile is normalised and staged in LDS; a routed tile's staged
// output goes to HBM during the next tile's first kv step (c.pending), a window tile's at once.
template <int NG, bool LOCAL, bool FUSED, bool CLIP, typename RequestNext, typename DescribeNext>
__device__ __forceinline__ void flash_tile(const FlashArgs& a, char* lds, const TileDesc& cur,
                                           TileDesc& next, bool has_next, RequestNext&& request_next,
                                           DescribeNext&& describe_next, FlashCarry& c) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = wave >> 2, w4 = wave & 3;  // grp 0 = early, 1 = late
  const int qc = lane & 31, hf = lane >> 5;
  const int srow = w4 * 32 + qc;             // row inside the group's 128-row half tile
  using Lds = FlashLds<NG>;
  constexpr int kStagesK = Lds::kStagesK, kStagesV = Lds::kStagesV, BPW = Lds::kBlocksPerWave;
  bf16_t* const ldsV = reinterpret_cast<bf16_t*>(lds + Lds::kV);
  bf16_t* const ldsK = reinterpret_cast<bf16_t*>(lds + Lds::kK);

  // Direct global -> LDS staging of one (K, V^T) tile pair in 1 KB blocks (4 K rows or 8 V^T rows
  // each); lane L of a block lands at byte 16*L.
  // Per-lane byte offsets are loop-invariant 32-bit values; the kv head and the tile position
  // go into the wave-uniform base pointer.
  uint32_t koff[BPW], voff[BPW];
#pragma unroll
  for (int i = 0; i < BPW; ++i) {
    const int blk = wave * BPW + i;
    const int row = blk * 4 + (lane >> 4), pc = lane & 15, gp = pc ^ (row & 15);
    koff[i] = (uint32_t)((row * a.kvst + gp * 8) * sizeof(bf16_t));
    const int d = blk * 8 + (lane >> 3), pv = lane & 7, gv = pv ^ ((d >> 1) & 7);
    voff[i] = (uint32_t)((d * a.Lp + gv * 8) * sizeof(bf16_t));
  }
  // wavefront w fills blocks w*BPW .. w*BPW + BPW-1 of both tiles
  auto stage = [&](int kvh, int64_t t0, int kb, int vb) {
    const char* kbase = reinterpret_cast<const char*>(a.K + (int64_t)kvh * a.kvsh + t0 * a.kvst);
    const char* vbase = reinterpret_cast<const char*>(a.Vt + (int64_t)kvh * HD * a.Lp + t0);
#pragma unroll
    for (int i = 0; i < BPW; ++i) {
      uint32_t off = koff[i];
      if (LOCAL || CLIP) {  // rows past the end of the sequence re-read the last row (masked later)
        const int row = (wave * BPW + i) * 4 + (lane >> 4);
        if (t0 + row >= a.L) off -= (uint32_t)((t0 + row - (a.L - 1)) * a.kvst * sizeof(bf16_t));
      }
      __builtin_amdgcn_global_load_lds(SL_GLOBAL_PTR(kbase + off),
                                       SL_LDS_PTR(ldsK + kb * kStageElems + (wave * BPW + i) * 512), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < BPW; ++i)
      __builtin_amdgcn_global_load_lds(SL_GLOBAL_PTR(vbase + voff[i]),
                                       SL_LDS_PTR(ldsV + vb * kStageElems + (wave * BPW + i) * 512), 16, 0, 0);
  };
  // Q row of a lane's column, as the B operand of S^T = K Q^T
  auto load_q = [&](int64_t q_off) {
    const bf16_t* qp = a.Q + q_off;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) c.qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16 + hf * 8);
  };
  if (!c.primed) {
    stage(cur.kv, cur.kv_begin, c.kb, c.vb);
    load_q(cur.q_off);
  }

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;  // m in log2 units of the scaled logit
  bf16x8 pb[4];                  // P^T fragments; the late group carries them to the next kv tile
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int e = 0; e < 8; ++e) pb[ks][e] = (__bf16)0.f;

  const int krow = perm_row(qc);
  const int kswz = krow & 15;      // swizzle key of this lane's K rows (32*sub does not change it)
  const int vswz = (qc >> 1) & 7;  // swizzle key of this lane's V^T rows (32*dt does not change it)
  const float sc = a.scale_log2e;

  // S^T = K Q^T (two 32-row halves of the tile), mask, running maximum, exponentials -> pb.
  // LDS fragment reads run four MFMAs ahead (0x100 = LDS read, 0x008 = MFMA).
  auto qk_softmax = [&](const bf16_t* kt, int64_t t0) {
    f32x16 s[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const bf16x8 ka = *reinterpret_cast<const bf16x8*>(
            &kt[(32 * sub + krow) * HD + (((2 * kk + hf) ^ kswz) << 3)]);
        s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, c.qf[kk], s[sub], 0, 0, 0);
      }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int i = 0; i < 12; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    // The softmax arithmetic below competes for issue slots with the MFMA stream of the SIMD's
    // other wavefront; that one needs a slot every 32 cycles, this one needs most of them.
    __builtin_amdgcn_s_setprio(3);

    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (LOCAL || CLIP) {  // per-row range: the causal window, or a span clipped behind a lower one
          const int64_t t = t0 + 32 * sub + 16 * (r >> 3) + 8 * hf + (r & 7);
          s[sub][r] = (t <= cur.i_q && t >= cur.lo_q) ? s[sub][r] : -INFINITY;
        }
        mx = fmaxf(mx, s[sub][r]);
      }
    mx = pair_max(mx) * sc;
    // Lazy rescale, decided per column: a column's running maximum only moves when that column
    // grew by more than 2^8; until then its exponentials are taken against the old maximum
    // (p <= 256).  The branch is per wavefront, the arithmetic of a column does not depend on the
    // columns it shares the wavefront with (so a row's result does not depend on its tile-mates).
    const bool grow = mx > m + 8.f || (m == -INFINITY && mx > -INFINITY);
    if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
      const float alpha = grow ? fast_exp2(m - mx) : 1.f;  // m = -inf: 0, and l and o are still 0
      m = grow ? mx : m;
      l *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
    const float nm = m > -INFINITY ? -m : 0.f;  // whole column masked so far: exponentials are 0 anyway
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      f32x8 p;
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = fast_exp2(fmaf(s[ks >> 1][8 * (ks & 1) + e], sc, nm));
      pb[ks] = __builtin_convertvector(p, bf16x8);
      // the row sum is taken over the rounded weights, the ones the PV product uses
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const bf16x2 pr = {pb[ks][e], pb[ks][e + 1]};
        const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
        l = __builtin_amdgcn_fdot2_f32_bf16(pr, one, l, false);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // O^T += V^T P^T with the P^T fragments in pb
  auto pv = [&](const bf16_t* vt) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const bf16x8 va = *reinterpret_cast<const bf16x8*>(
            &vt[(32 * dt + qc) * TN + (((2 * ks + hf) ^ vswz) << 3)]);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[ks], o[dt], 0, 0, 0);
      }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 1);
#pragma unroll
    for (int i = 0; i < 12; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 1);
  };

  int kb = c.kb, vb = c.vb, vb_prev = c.vb;
  for (int64_t t0 = cur.kv_begin; t0 < cur.kv_end; t0 += TN) {
    // After the barrier the tile of this iteration is visible to every wavefront, every wavefront
    // is done with the K stage of the previous tile and the late group with the V^T stage before
    // that: exactly the stages that the next tile goes into.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    const int kb1 = kb == kStagesK - 1 ? 0 : kb + 1, vb1 = vb == kStagesV - 1 ? 0 : vb + 1;
    if (NG == 2 && !LOCAL && c.pending) {
      // the previous tile's output: written out here, a step after it was staged, so that the wait
      // at the top of this tile did not have to cover its stores
      flush_routed_output(a, lds, grp, w4, lane);
      c.pending = false;
    }
    if (t0 + TN < cur.kv_end) stage(cur.kv, t0 + TN, kb1, vb1);
    if (NG == 2 && has_next && t0 == cur.kv_begin) request_next();
    if (grp == 0) {
      qk_softmax(ldsK + kb * kStageElems, t0);
      pv(ldsV + vb * kStageElems);
    } else {
      if (t0 > cur.kv_begin) pv(ldsV + vb_prev * kStageElems);
      qk_softmax(ldsK + kb * kStageElems, t0);
    }
    vb_prev = vb;
    kb = kb1;
    vb = vb1;
  }
  // Every wavefront is past its last QK: all K stages and the Q fragments are dead, and so is
  // every V^T stage except the last tile's (the late group still owes its PV).  Request the next
  // tile's first stage and Q fragments now; they land while this tile is written out.
  __syncthreads();
  c.kb = kb;
  c.vb = vb;
  c.primed = NG == 2 && has_next;  // NG = 1: the output region lies over the stages, nothing is fetched ahead
  if (NG == 2 && has_next) {
    next = describe_next();
    stage(next.kv, next.kv_begin, kb, vb);
    load_q(next.q_off);
  }
  // From here to the end of the tile the late group is the critical path (it still owes a PV):
  // its wavefronts go first wherever both groups want an issue slot.
  if (NG == 2 && grp == 1) __builtin_amdgcn_s_setprio(2);
  if (grp == 1) pv(ldsV + vb_prev * kStageElems);  // the late group's last PV

  // epilogue, wavefront-local (no workgroup barrier): normalise, stage the wavefront's 32 rows as
  // [row][d] bf16 in its own slice of the group's LDS region (swizzled 16-byte pieces), then
  // write 16 lanes per row, 16 bytes per lane.  LDS operations of one wavefront complete in
  // issue order, so the reads below see the writes of the other lanes.
  const float lt = pair_sum(l);
  const float inv = 1.f / lt;
  bf16_t* const ost = reinterpret_cast<bf16_t*>(lds + Lds::kOut) + grp * TG * HD;
  int64_t* const row_out = reinterpret_cast<int64_t*>(lds + Lds::kRowOut) + grp * TG;
  float* const row_lse = reinterpret_cast<float*>(lds + Lds::kRowLse) + grp * TG;
  if (hf == 0) {
    row_lse[srow] = (m + __log2f(lt)) * kLn2;
    row_out[srow] = cur.row_out;
  }
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int unit = (4 * dt + g4) ^ (srow & 15);
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = o[dt][4 * g4 + e] * inv;
      const bf16x4 w = __builtin_convertvector(v, bf16x4);
      *reinterpret_cast<bf16x4*>(&ost[srow * HD + unit * 8 + 4 * hf]) = w;
    }
  __builtin_amdgcn_wave_barrier();
  if constexpr (FUSED) {
    // Local-window tile with the merge fused in (topk <= 8): the lane that would store 16 bytes
    // of the window's partial instead loads the same 16 bytes of the row's routed partials
    // (written by the routed kernel, which ran before on the stream), does the log-sum-exp merge
    // and stores the final output.  Every load is issued before the first dependent use; slots
    // that take no part may hold anything and are discarded by selects, never by arithmetic.
    const int topk = a.topk, nslot = topk + 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      int64_t outs[4];
      int js[4][8];
      float ls[4][8];
      uint4 ov[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int row = w4 * 32 + (half * 4 + u) * 4 + (lane >> 4), piece = lane & 15;
        outs[u] = row_out[row];
        const int64_t rg = outs[u] >= 0 ? outs[u] : 0;
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
          const bool in = sl < topk;
          js[u][sl] = in ? a.idx[rg * topk + sl] : -1;
          ls[u][sl] = in ? a.part_lse[rg * nslot + sl] : 0.f;
          ov[u][sl] = in ? load16(a.part_o + (rg * nslot + sl) * HD + piece * 8) : make_uint4(0, 0, 0, 0);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int row = w4 * 32 + (half * 4 + u) * 4 + (lane >> 4), piece = lane & 15;
        const int cq = (int)((a.q_pos0 + (outs[u] - cur.row_base)) / a.A);
        const float lw = row_lse[row];
        float M = lw;
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
          // a slot takes part if its span is a candidate and no earlier slot lists the same span
          bool ok = js[u][sl] >= 0 && js[u][sl] < cq;
#pragma unroll
          for (int v = 0; v < sl; ++v) ok = ok && js[u][v] != js[u][sl];
          ls[u][sl] = ok ? ls[u][sl] : -INFINITY;
          M = fmaxf(M, ls[u][sl]);
        }
        float acc[8], f[8];
        float wsum = __expf(lw - M);
        Elem<bf16_t>::unpack(*reinterpret_cast<const uint4*>(&ost[row * HD + ((piece ^ (row & 15)) << 3)]), f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = wsum * f[e];
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
          const bool ok = ls[u][sl] > -INFINITY;
          const float w = ok ? __expf(ls[u][sl] - M) : 0.f;
          wsum += w;
          Elem<bf16_t>::unpack(ok ? ov[u][sl] : make_uint4(0, 0, 0, 0), f);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, f[e], acc[e]);
        }
        const float winv = 1.f / wsum;
        uint4 res;
        res.x = (uint32_t)f32_to_bf16(acc[0] * winv) | ((uint32_t)f32_to_bf16(acc[1] * winv) << 16);
        res.y = (uint32_t)f32_to_bf16(acc[2] * winv) | ((uint32_t)f32_to_bf16(acc[3] * winv) << 16);
        res.z = (uint32_t)f32_to_bf16(acc[4] * winv) | ((uint32_t)f32_to_bf16(acc[5] * winv) << 16);
        res.w = (uint32_t)f32_to_bf16(acc[6] * winv) | ((uint32_t)f32_to_bf16(acc[7] * winv) << 16);
        if (outs[u] >= 0) {
          *reinterpret_cast<uint4*>(a.O + outs[u] * HD + piece * 8) = res;
          if (piece == 0) a.LSE[outs[u]] = M + __logf(wsum);
        }
      }
    }
  } else if (NG == 2 && !LOCAL) {
    c.pending = true;  // written out during the next tile's first kv step, or by the caller after the last tile
  } else {
    // Every LDS read comes before the first store, and the values are pinned there: the compiler
    // orders an LDS read after all outstanding vector-memory operations once direct global->LDS
    // loads are in flight (the next tile's), so a read between two stores would wait for the
    // earlier store to be acknowledged.
    int64_t outs[8];
    uint4 vals[8];
    float lses[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = w4 * 32 + u * 4 + (lane >> 4), piece = lane & 15;
      outs[u] = row_out[row];
      lses[u] = row_lse[row];
      vals[u] = *reinterpret_cast<const uint4*>(&ost[row * HD + ((piece ^ (row & 15)) << 3)]);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      asm volatile("" : "+v"(vals[u].x), "+v"(vals[u].y), "+v"(vals[u].z), "+v"(vals[u].w), "+v"(lses[u]),
                   "+v"(outs[u]));
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int piece = lane & 15;
      if (outs[u] >= 0) {
        *reinterpret_cast<uint4*>(a.part_o + outs[u] * HD + piece * 8) = vals[u];
        if (piece == 0) a.part_lse[outs[u]] = lses[u];
      }
    }
  }
  __builtin_amdgcn_s_setprio(0);
  __builtin_amdgcn_wave_barrier();
  // No trailing barrier: a wavefront's output slice is private to it, and the K/V stages are
  // handed over through c.kb / c.vb.
}

// Routed spans: persistent workgroups walk the tile list.  XCD x (workgroups with
// blockIdx % 8 == x) owns the contiguous chunk [x*T/8, (x+1)*T/8) of the tile list; its
// workgroups walk the chunk interleaved, so at any moment they sit on neighbouring tiles -- the
// same one or two buckets -- and share the span through that XCD's L2.  The record and the item
// of a workgroup's next tile are fetched while its current tile is computed.
// CLIP (overlapping spans, anchor spacing A < S, joint softmax): a row's range in span j starts behind
// the end of the nearest lower span that the row lists, so that every token of the union counts once.
template <bool CLIP>
__global__ __launch_bounds__(FlashLds<2>::kThreads, 1) void span_flash_routed_kernel(const FlashArgs a) {
  extern __shared__ __align__(16) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qrow = (wave >> 2) * TG + (wave & 3) * 32 + (lane & 31);
  const int64_t T = a.tile_off[a.Hq / a.G * a.n];
  const int NWL = gridDim.x / 8;  // workgroups per XCD (the grid is a multiple of 8)
  const int xcd = blockIdx.x % 8, wl = blockIdx.x / 8;
  const int64_t c_begin = T * xcd / 8, c_end = T * (xcd + 1) / 8;
  const int64_t t_begin = c_begin + wl, t_end = c_end;
  if (t_begin >= t_end) return;

  auto describe = [&](const int4& info, int item) {
    TileDesc d;
    d.kv = info.x / a.n;
    const int j = info.x % a.n;
    d.kv_end = (int64_t)(j + 1) * a.A;
    d.kv_begin = d.kv_end - a.S > 0 ? d.kv_end - a.S : 0;
    const int rowid = item >> 5, slot = item & 31;
    const int hl = rowid / (int)a.Lq;
    const int64_t r = rowid - (int64_t)hl * a.Lq;
    const int h = d.kv * a.G + hl;
    d.q_off = h * a.qsh + r * a.qst;
    d.row_out = qrow < info.z ? ((int64_t)h * a.Lq + r) * (a.topk + 1) + slot : -1;
    d.i_q = d.kv_end;
    d.lo_q = 0;
    if (CLIP) {
      const int64_t c = (a.q_pos0 + r) / a.A;
      const int32_t* irow = a.idx + ((int64_t)h * a.Lq + r) * a.topk;
      for (int s2 = 0; s2 < a.topk; ++s2) {
        const int64_t jj = irow[s2];
        if (jj >= 0 && jj < c && jj < j && (jj + 1) * a.A > d.lo_q) d.lo_q = (jj + 1) * a.A;
      }
    }
    d.row_base = 0;
    return d;
  };
  FlashCarry carry;
  carry.kb = carry.vb = 0;
  carry.primed = false;
  carry.pending = false;
  // The record and the items of a workgroup's next tile are requested during the current tile's
  // first kv step as direct global->LDS loads into the wavefront's own 512 bytes (the items of tile t sit
  // at t*TM, so the two do not depend on each other) and read back at its tail.
  int* const ahead = reinterpret_cast<int*>(lds + FlashLds<2>::kAhead) + wave * 128;
  const int4 info0 = a.tile_info[t_begin];
  TileDesc cur = describe(info0, a.items[t_begin * TM + qrow]);
  for (int64_t t = t_begin; t < t_end; t += NWL) {
    const bool has_next = t + NWL < t_end;
    TileDesc nxt = cur;
    flash_tile<2, false, false, CLIP>(
        a, lds, cur, nxt, has_next,
        [&] {
          const int* rec = reinterpret_cast<const int*>(a.tile_info + (t + NWL)) + (lane & 3);
          const int* itm = a.items + (t + NWL) * TM + wave * 32 + (lane & 31);
          __builtin_amdgcn_global_load_lds(SL_GLOBAL_PTR(rec), SL_LDS_PTR(ahead), 4, 0, 0);
          __builtin_amdgcn_global_load_lds(SL_GLOBAL_PTR(itm), SL_LDS_PTR(ahead + 64), 4, 0, 0);
        },
        [&] {
          const int4 ninfo = make_int4(ahead[0], ahead[1], ahead[2], 0);
          return describe(ninfo, ahead[64 + lane]);
        },
        carry);
    cur = nxt;
  }
  // the last tile's output (its epilogue ended with the wavefront's own LDS writes)
  if (carry.pending) flush_routed_output(a, lds, wave >> 2, wave & 3, lane);
}

// The paper's geometry: routed tiles of a (kv head, end block) bucket.  Every row of a tile has
// its own token range [lo, hi) (hi inside the bucket's block); the tile walks the kv range from
// the lowest lo to the highest hi of its rows (rounded to whole 64-token tiles) with per-row masks.
__global__ __launch_bounds__(FlashLds<2>::kThreads, 1) void span_flash_anchor_kernel(const FlashArgs a) {
  extern __shared__ __align__(16) char lds[];
  __shared__ int64_t s_lo[8], s_hi[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qrow = (wave >> 2) * TG + (wave & 3) * 32 + (lane & 31);
  const int64_t T = a.tile_off[a.Hq / a.G * a.n];
  const int NWL = gridDim.x / 8;
  const int xcd = blockIdx.x % 8, wl = blockIdx.x / 8;
  const int64_t c_begin = T * xcd / 8, c_end = T * (xcd + 1) / 8;
  const int64_t t_begin = c_begin + wl, t_end = c_end;
  if (t_begin >= t_end) return;

  // all threads call (two barriers inside)
  auto describe = [&](const int4& info, int item) {
    TileDesc d;
    d.kv = info.x / a.n;
    const int rowid = item >> 5, slot = item & 31;
    const int hl = rowid / (int)a.Lq;
    const int64_t r = rowid - (int64_t)hl * a.Lq;
    const int h = d.kv * a.G + hl;
    const int64_t i = a.q_pos0 + r;
    const bool real = qrow < info.z;
    const int64_t t = a.idx[((int64_t)h * a.Lq + r) * a.topk + slot];
    const AnchorSpan sp = anchor_span_of(i, t, span_base_length(i, a.aroot), a.window, a.ab, a.af);
    d.q_off = h * a.qsh + r * a.qst;
    d.row_out = real ? ((int64_t)h * a.Lq + r) * (a.topk + 1) + slot : -1;
    d.lo_q = sp.lo;
    d.i_q = sp.hi - 1;
    d.row_base = 0;
    // the tile's kv range: from the lowest lo to the highest hi of its rows
    int64_t lo = real && sp.hi > sp.lo ? sp.lo : INT64_MAX, hi = real && sp.hi > sp.lo ? sp.hi : 0;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const int64_t lo2 = __shfl_xor(lo, off, 64), hi2 = __shfl_xor(hi, off, 64);
      lo = lo2 < lo ? lo2 : lo;
      hi = hi2 > hi ? hi2 : hi;
    }
    __syncthreads();  // earlier readers of s_lo / s_hi are done
    if (lane == 0) {
      s_lo[wave] = lo;
      s_hi[wave] = hi;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      lo = s_lo[w] < lo ? s_lo[w] : lo;
      hi = s_hi[w] > hi ? s_hi[w] : hi;
    }
    if (hi <= lo) lo = hi = 0;  // cannot happen for a tile with items; keeps the range sane
    d.kv_begin = lo / TN * TN;
    d.kv_end = (hi + TN - 1) / TN * TN;
    return d;
  };
  FlashCarry carry;
  carry.kb = carry.vb = 0;
  carry.primed = false;
  carry.pending = false;
  int* const ahead = reinterpret_cast<int*>(lds + FlashLds<2>::kAhead) + wave * 128;
  const int4 info0 = a.tile_info[t_begin];
  TileDesc cur = describe(info0, a.items[t_begin * TM + qrow]);
  for (int64_t t = t_begin; t < t_end; t += NWL) {
    const bool has_next = t + NWL < t_end;
    TileDesc nxt = cur;
    flash_tile<2, false, false, true>(
        a, lds, cur, nxt, has_next,
        [&] {
          const int* rec = reinterpret_cast<const int*>(a.tile_info + (t + NWL)) + (lane & 3);
          const int* itm = a.items + (t + NWL) * TM + wave * 32 + (lane & 31);
          __builtin_amdgcn_global_load_lds(SL_GLOBAL_PTR(rec), SL_LDS_PTR(ahead), 4, 0, 0);
          __builtin_amdgcn_global_load_lds(SL_GLOBAL_PTR(itm), SL_LDS_PTR(ahead + 64), 4, 0, 0);
        },
        [&] {
          const int4 ninfo = make_int4(ahead[0], ahead[1], ahead[2], 0);
          return describe(ninfo, ahead[64 + lane]);
        },
        carry);
    cur = nxt;
  }
  if (carry.pending) flush_routed_output(a, lds, wave >> 2, wave & 3, lane);
}

// Row tiles of the local-window kernel and their grouping into chunks of `tps` tiles (the tiles
// of one span when S is a multiple of the tile height).
struct LocalMap {
  int tiles_per_head, tps, chunks;
};
__host__ __device__ inline LocalMap local_map(int64_t Lq, int S) {
  LocalMap m;
  m.tiles_per_head = (int)((Lq + FlashLds<1>::kRows - 1) / FlashLds<1>::kRows);
  m.tps = S / FlashLds<1>::kRows > 0 ? S / FlashLds<1>::kRows : 1;
  m.chunks = (m.tiles_per_head + m.tps - 1) / m.tps;
  return m;
}
// Blocks to launch: 8 x the largest per-XCD share.
inline unsigned local_grid(int64_t Lq, int S, int Hkv, int G) {
  const LocalMap m = local_map(Lq, S);
  int best = 0;
  for (int x = 0; x < 8; ++x) {
    const int cx = (m.chunks - x + 7) / 8;
    const bool lx = m.chunks > 0 && (m.chunks - 1) % 8 == x;
    const int tx = cx * m.tps - (lx ? m.chunks * m.tps - m.tiles_per_head : 0);
    best = tx > best ? tx : best;
  }
  return (unsigned)(8 * Hkv * best * G);
}

// Local window [c*S, i]: regular 128-row tiles of one head with the causal / window mask.
// FUSED = false: writes the window's partial into the row's last slot (a merge kernel follows).
// FUSED = true (joint softmax, topk <= 8): merges the row's routed partials in the epilogue and
// writes the final output, which takes the merge's HBM traffic off the critical path of a
// separate kernel and saves the window partial's round trip.
template <bool FUSED>
__global__ __launch_bounds__(FlashLds<1>::kThreads, 2) void span_flash_local_kernel(const FlashArgs a) {
  extern __shared__ __align__(16) char lds[];
  constexpr int TML = FlashLds<1>::kRows;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qrow = wave * 32 + (lane & 31);
  // Workgroup -> (head, row tile), XCD-aware: blocks are dealt round-robin to the 8 XCDs, each
  // with its own L2.  A run of `tps` consecutive row tiles (one span's worth) goes to one XCD,
  // and inside an XCD the G query heads of a kv head take the same row tile back to back, so the
  // window's K/V tiles are fetched from HBM about once instead of once per head and row tile.
  const LocalMap lm = local_map(a.Lq, a.A);
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int chunks_x = (lm.chunks - xcd + 7) / 8;                 // chunks xcd, xcd+8, ... of a kv head
  const bool has_last = lm.chunks > 0 && (lm.chunks - 1) % 8 == xcd;  // the only chunk that may be short
  const int tiles_x = chunks_x * lm.tps - (has_last ? lm.chunks * lm.tps - lm.tiles_per_head : 0);
  if (slot >= (a.Hq / a.G) * tiles_x * a.G) return;  // uniform: the grid is padded to 8 * the largest share
  const int kvh = slot / (tiles_x * a.G), rem = slot % (tiles_x * a.G);
  const int tile_local = rem / a.G, g = rem % a.G;
  const int tile = (xcd + 8 * (tile_local / lm.tps)) * lm.tps + tile_local % lm.tps;
  const int h = kvh * a.G + g;
  const int64_t r0 = (int64_t)tile * TML;
  const int64_t r = r0 + qrow;
  const int64_t rc = r < a.Lq ? r : a.Lq - 1;
  TileDesc d;
  d.kv = h / a.G;
  d.q_off = h * a.qsh + rc * a.qst;
  d.row_base = (int64_t)h * a.Lq;
  if (FUSED) d.row_out = r < a.Lq ? d.row_base + r : -1;
  else d.row_out = r < a.Lq ? (d.row_base + r) * (a.topk + 1) + a.topk : -1;
  d.i_q = a.q_pos0 + rc;
  const int64_t i_first = a.q_pos0 + r0;
  const int64_t i_last = min(a.q_pos0 + r0 + TML - 1, a.q_pos0 + a.Lq - 1);
  if (a.window > 0) {  // the paper's geometry: a sliding window [i - window + 1, i] per row
    d.lo_q = d.i_q - a.window + 1 > 0 ? d.i_q - a.window + 1 : 0;
    const int64_t first_lo = i_first - a.window + 1 > 0 ? i_first - a.window + 1 : 0;
    d.kv_begin = first_lo / TN * TN;
  } else {
    d.lo_q = (d.i_q / a.A) * a.A;
    d.kv_begin = (i_first / a.A) * a.A;
  }
  d.kv_end = d.kv_begin + ((i_last - d.kv_begin) / TN + 1) * TN;
  FlashCarry carry;
  carry.kb = carry.vb = 0;
  carry.primed = false;
  carry.pending = false;
  TileDesc unused = d;
  flash_tile<1, true, FUSED, false>(a, lds, d, unused, false, [] {}, [&] { return d; }, carry);
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
    ov[s] = ok ? load16_stream(orow + (int64_t)s * HD) : make_uint4(0, 0, 0, 0);
  }
  ls[KMAX] = lrow[topk];
  ov[KMAX] = load16_stream(orow + (int64_t)topk * HD);

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


// Combination form of the merge (Section 3.4, eq. (5)-(6); Algorithm 1): per valid slot t,
// A_t = log-sum-exp merge of the slot's partial with the local window's partial (the attention
// over span t and the window with its own softmax); O = sum_t alpha_t A_t with alpha = softmax of
// the slots' search scores; no valid slot: the window's partial.
// ANCHOR: the paper's geometry.  idx holds anchor tokens, a slot is valid if its anchor is one of
// the row's (0 <= t <= i); a valid slot whose span minus the window is empty has lse = -inf and
// A_t is then the window's attention alone.
template <int KMAX, bool ANCHOR>
__global__ __launch_bounds__(256) void merge_combined_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ gate,
    const bf16_t* __restrict__ part_o, const float* __restrict__ part_lse, bf16_t* __restrict__ O,
    int64_t rows, int64_t Lq, int64_t q_pos0, int S, int topk) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int piece = threadIdx.x & 15;
  if (row >= rows) return;
  const int64_t r = row % Lq;
  const int64_t limit = ANCHOR ? q_pos0 + r + 1 : (q_pos0 + r) / S;  // valid entries lie in [0, limit)
  const int nslot = topk + 1;
  const int32_t* irow = idx + row * topk;
  const float* grow = gate + row * topk;
  const float* lrow = part_lse + row * nslot;
  const bf16_t* orow = part_o + row * nslot * HD + piece * 8;

  int js[KMAX];
  float ls[KMAX], gs[KMAX];
  uint4 ov[KMAX + 1];
#pragma unroll
  for (int s = 0; s < KMAX; ++s) js[s] = s < topk ? irow[s] : -1;
  float gmax = -INFINITY;
  unsigned okmask = 0u;
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    bool ok = js[s] >= 0 && js[s] < limit;
    if (!ANCHOR) {
#pragma unroll
      for (int u = 0; u < s; ++u) ok = ok && js[u] != js[s];
    }
    ls[s] = ok ? lrow[s] : -INFINITY;
    gs[s] = ok ? grow[s] : -INFINITY;
    ov[s] = (ok && ls[s] > -INFINITY) ? load16_stream(orow + (int64_t)s * HD) : make_uint4(0, 0, 0, 0);
    gmax = fmaxf(gmax, gs[s]);
    okmask |= ok ? (1u << s) : 0u;
  }
  const float lw = lrow[topk];
  ov[KMAX] = load16_stream(orow + (int64_t)topk * HD);

  float acc[8], fw[8], f[8];
  Elem<bf16_t>::unpack(ov[KMAX], fw);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  float asum = 0.f;
#pragma unroll
  for (int s = 0; s < KMAX; ++s) {
    if (okmask & (1u << s)) {  // valid slot
      const float M = fmaxf(ls[s], lw);
      const float wa = ls[s] > -INFINITY ? __expf(ls[s] - M) : 0.f, wb = __expf(lw - M);
      const float a = __expf(gs[s] - gmax);
      const float fa = a * wa / (wa + wb), fb = a * wb / (wa + wb);
      asum += a;
      Elem<bf16_t>::unpack(ov[s], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(fa, f[e], fmaf(fb, fw[e], acc[e]));
    }
  }
  const bool any = asum > 0.f;
  const float inv = any ? 1.f / asum : 1.f;
  uint4 res;
  float o8[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o8[e] = (any ? acc[e] : fw[e]) * inv;
  res.x = (uint32_t)f32_to_bf16(o8[0]) | ((uint32_t)f32_to_bf16(o8[1]) << 16);
  res.y = (uint32_t)f32_to_bf16(o8[2]) | ((uint32_t)f32_to_bf16(o8[3]) << 16);
  res.z = (uint32_t)f32_to_bf16(o8[4]) | ((uint32_t)f32_to_bf16(o8[5]) << 16);
  res.w = (uint32_t)f32_to_bf16(o8[6]) | ((uint32_t)f32_to_bf16(o8[7]) << 16);
  *reinterpret_cast<uint4*>(O + row * HD + piece * 8) = res;
}

// ------------------------------------------------------------------ workspace carving
struct MfmaWs {
  size_t vt, counts, blk_cnt, item_off, tile_off, cursor, tile_info, items, part_lse, part_o, total;
  int chunks;
  int64_t Lp;
  int B, max_tiles;
  int64_t max_items;
};

// Per-device facts, looked up on the first call with that device current: the grid of the
// persistent kernel (one resident workgroup of eight wavefronts per compute unit) and whether the
// flash kernels were granted more dynamic LDS than the 64 KB a kernel gets by default.
struct DeviceSetup {
  int grid = 0;     // 0 = not looked up yet
  bool lds_ok = false;
};
constexpr int kMaxDevices = 64;
std::mutex g_setup_mu;
DeviceSetup g_setup[kMaxDevices];

bool device_setup(DeviceSetup* out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
  std::lock_guard<std::mutex> lock(g_setup_mu);
  DeviceSetup& d = g_setup[dev];
  if (d.grid == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    d.lds_ok =
        hipFuncSetAttribute(reinterpret_cast<const void*>(span_flash_routed_kernel<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FlashLds<2>::kBytes) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(span_flash_routed_kernel<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FlashLds<2>::kBytes) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(span_flash_anchor_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FlashLds<2>::kBytes) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(span_flash_local_kernel<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FlashLds<1>::kBytes) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(span_flash_local_kernel<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FlashLds<1>::kBytes) == hipSuccess;
    d.grid = (cus + 7) / 8 * 8;
  }
  *out = d;
  return true;
}

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
  w.chunks = (int)((pb.Lq + kBucketRows - 1) / kBucketRows);
  w.blk_cnt = take((size_t)pb.Hq * w.chunks * pb.n * sizeof(int));
  w.item_off = take((size_t)(w.B + 1) * sizeof(int));
  w.tile_off = take((size_t)(w.B + 1) * sizeof(int));
  w.cursor = take((size_t)w.B * sizeof(int));
  w.tile_info = take((size_t)w.max_tiles * sizeof(int4));
  w.items = take((size_t)w.max_tiles * TM * sizeof(int));  // tile by tile, TM entries each
  const size_t nparts = (size_t)pb.Hq * pb.Lq * (pb.topk + 1);  // routed slots + the local window
  w.part_lse = take(nparts * sizeof(float));
  w.part_o = take(nparts * HD * sizeof(bf16_t));
  w.total = off;
  return w;
}

}  // namespace

bool prefill_attention_mfma_supported(const Problem& pb) {
  return pb.dtype == SL_BF16 && pb.D == HD && pb.S % TN == 0 && pb.A % TN == 0 && pb.n <= 4096 &&
         (int64_t)pb.G * pb.Lq < ((int64_t)1 << 26) &&  // item = (row id << 5) | slot
         // staging uses 32-bit byte offsets inside one kv head's V^T and inside a 64-row K tile
         (int64_t)HD * (int64_t)align_up((size_t)pb.L, 64) * 2 < ((int64_t)1 << 32) &&
         64 * pb.kvst * 2 < ((int64_t)1 << 31) &&
         (int64_t)pb.Hq * pb.Lq * (pb.topk + 1) < ((int64_t)1 << 31) &&
         // 32-bit positions in the tile-by-tile item list
         (int64_t)pb.Hq * pb.Lq * pb.topk + ((int64_t)pb.Hkv * pb.n + 1) * TM < ((int64_t)1 << 31) &&
         // row_q holds 32-bit element offsets into Q
         (int64_t)pb.Hq * pb.qsh + pb.Lq * pb.qst < ((int64_t)1 << 31);
}

size_t prefill_attention_mfma_ws_bytes(const Problem& pb) { return carve(pb).total; }

sl_status prefill_attention_mfma(const Problem& pb, const void* Q, const void* K, const void* V,
                                 const int32_t* idx, void* O, float* LSE, void* ws,
                                 hipStream_t st) {
  const MfmaWs w = carve(pb);
  DeviceSetup dev;
  if (!device_setup(&dev) || !dev.lds_ok) return SL_ERR_LAUNCH;
  char* base = static_cast<char*>(ws);
  bf16_t* Vt = reinterpret_cast<bf16_t*>(base + w.vt);
  int* counts = reinterpret_cast<int*>(base + w.counts);
  int* blk_cnt = reinterpret_cast<int*>(base + w.blk_cnt);
  int* item_off = reinterpret_cast<int*>(base + w.item_off);
  int* tile_off = reinterpret_cast<int*>(base + w.tile_off);
  int* cursor = reinterpret_cast<int*>(base + w.cursor);
  int4* tile_info = reinterpret_cast<int4*>(base + w.tile_info);
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
  a.tile_info = tile_info;
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
  a.A = pb.A;
  a.window = 0;
  a.ab = a.af = 0;
  a.aroot = 2;
  a.E = 0;
  a.topk = pb.topk;
  a.n = n;
  a.scale_log2e = pb.scale * kLog2e;
  a.qsh = pb.qsh;
  a.qst = pb.qst;
  a.kvsh = pb.kvsh;
  a.kvst = pb.kvst;

  if (pb.topk > 0) {
    const dim3 bgrid((unsigned)w.chunks, pb.Hq);
    hipLaunchKernelGGL(bucket_kernel<false>, bgrid, dim3(256), (size_t)n * sizeof(int), st, idx,
                       blk_cnt, cursor, items, pb.Lq, pb.q_pos0, pb.G, pb.A, pb.topk, n);
    hipLaunchKernelGGL(bucket_block_scan_kernel, dim3((n + 31) / 32, pb.Hkv), dim3(256), 0, st, blk_cnt,
                       counts, pb.G * w.chunks, n);
    hipLaunchKernelGGL(bucket_scan_kernel, dim3(1), dim3(1024), 0, st, counts, item_off, tile_off,
                       cursor, w.B);
    hipLaunchKernelGGL(bucket_tiles_kernel, dim3(w.B), dim3(256), 0, st, tile_off, item_off, tile_info,
                       items);
    hipLaunchKernelGGL(bucket_kernel<true>, bgrid, dim3(256), (size_t)4 * n * sizeof(int), st, idx,
                       blk_cnt, cursor, items, pb.Lq, pb.q_pos0, pb.G, pb.A, pb.topk, n);
    if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
    if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
    if (pb.A < pb.S && !pb.combined)  // overlapping spans in one joint softmax: per-row clipping
      hipLaunchKernelGGL(span_flash_routed_kernel<true>, dim3(dev.grid), dim3(FlashLds<2>::kThreads),
                         FlashLds<2>::kBytes, st, a);
    else
      hipLaunchKernelGGL(span_flash_routed_kernel<false>, dim3(dev.grid), dim3(FlashLds<2>::kThreads),
                         FlashLds<2>::kBytes, st, a);
    if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  }
  const unsigned lgrid = local_grid(pb.Lq, pb.A, pb.Hkv, pb.G);
  if (!pb.combined && pb.topk <= 8) {  // the window kernel merges and writes the final output
    hipLaunchKernelGGL(span_flash_local_kernel<true>, dim3(lgrid), dim3(FlashLds<1>::kThreads),
                       FlashLds<1>::kBytes, st, a);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(span_flash_local_kernel<false>, dim3(lgrid), dim3(FlashLds<1>::kThreads),
                     FlashLds<1>::kBytes, st, a);
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  const dim3 mgrid((unsigned)((rows + 15) / 16));
#define SL_MERGE(KM)                                                                             \
  do {                                                                                           \
    if (pb.combined)                                                                                 \
      hipLaunchKernelGGL((merge_combined_kernel<KM, false>), mgrid, dim3(256), 0, st, idx, pb.gate, \
                         part_o, part_lse, a.O, rows, pb.Lq, pb.q_pos0, pb.A, pb.topk);          \
    else                                                                                         \
      hipLaunchKernelGGL(merge_partials_kernel<KM>, mgrid, dim3(256), 0, st, idx, part_o,        \
                         part_lse, a.O, LSE, rows, pb.Lq, pb.q_pos0, pb.A, pb.topk);             \
  } while (0)
  if (pb.topk == 0) SL_MERGE(1);
  else if (pb.topk <= 8) SL_MERGE(8);
  else if (pb.topk <= 16) SL_MERGE(16);
  else SL_MERGE(32);
#undef SL_MERGE
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

// ------------------------------------------------------------------ the paper's geometry on the matrix cores
namespace {

// End-block size E of the buckets: the smallest power-of-two multiple of 64 tokens that gives a
// bucket about two 256-row tiles of items on average, and at most 4096 blocks per kv head.
int anchor_block_tokens(const Problem& pb) {
  const int64_t items = (int64_t)pb.G * pb.Lq * (pb.topk > 0 ? pb.topk : 1);
  int64_t E = 64;
  while (E < 4096 && (items * E < 512 * pb.L || (pb.L + E - 1) / E > 4096)) E <<= 1;
  return (int)E;
}

Problem anchor_view(const Problem& pb) {
  Problem q = pb;
  q.A = anchor_block_tokens(pb);
  q.n = (pb.L + q.A - 1) / q.A;
  return q;
}

}  // namespace

bool prefill_anchor_mfma_supported(const Problem& pb, int64_t window) {
  const Problem q = anchor_view(pb);
  return window >= 1 && pb.topk >= 1 && pb.dtype == SL_BF16 && pb.D == HD && q.n <= 4096 &&
         (int64_t)pb.G * pb.Lq < ((int64_t)1 << 26) &&
         (int64_t)HD * (int64_t)align_up((size_t)pb.L, 64) * 2 < ((int64_t)1 << 32) &&
         64 * pb.kvst * 2 < ((int64_t)1 << 31) &&
         (int64_t)pb.Hq * pb.Lq * (pb.topk + 1) < ((int64_t)1 << 31) &&
         (int64_t)pb.Hq * pb.Lq * pb.topk + ((int64_t)pb.Hkv * q.n + 1) * TM < ((int64_t)1 << 31) &&
         (int64_t)pb.Hq * pb.qsh + pb.Lq * pb.qst < ((int64_t)1 << 31);
}

size_t prefill_anchor_mfma_ws_bytes(const Problem& pb) { return carve(anchor_view(pb)).total; }

// Span-attention and combination on the paper's geometry (Section 3.3-3.4, Algorithm 1), matrix-core
// form following Section 4.3's bucketing by key-block footprint: (row, slot) pairs are bucketed by
// the block that holds their span's last token, a bucket's rows share one sliding K/V range with
// per-row masks, the sliding window is a banded flash kernel, and the gated merge combines them.
sl_status prefill_anchor_attention_mfma(const Problem& pb, int64_t window, int b, int f, int root,
                                        const void* Q, const void* K, const void* V,
                                        const int32_t* anchors, void* O, void* ws, hipStream_t st) {
  const Problem q = anchor_view(pb);
  const MfmaWs w = carve(q);
  DeviceSetup dev;
  if (!device_setup(&dev) || !dev.lds_ok) return SL_ERR_LAUNCH;
  char* base = static_cast<char*>(ws);
  bf16_t* Vt = reinterpret_cast<bf16_t*>(base + w.vt);
  int* counts = reinterpret_cast<int*>(base + w.counts);
  int* blk_cnt = reinterpret_cast<int*>(base + w.blk_cnt);
  int* item_off = reinterpret_cast<int*>(base + w.item_off);
  int* tile_off = reinterpret_cast<int*>(base + w.tile_off);
  int* cursor = reinterpret_cast<int*>(base + w.cursor);
  int4* tile_info = reinterpret_cast<int4*>(base + w.tile_info);
  int* items = reinterpret_cast<int*>(base + w.items);
  float* part_lse = reinterpret_cast<float*>(base + w.part_lse);
  bf16_t* part_o = reinterpret_cast<bf16_t*>(base + w.part_o);
  const int n = (int)q.n;

  hipLaunchKernelGGL(transpose_v_kernel, dim3((unsigned)(w.Lp / 64), pb.Hkv), dim3(256), 0, st,
                     static_cast<const bf16_t*>(V), Vt, pb.L, w.Lp, pb.kvsh, pb.kvst);
  FlashArgs a;
  a.Q = static_cast<const bf16_t*>(Q);
  a.K = static_cast<const bf16_t*>(K);
  a.Vt = Vt;
  a.idx = anchors;
  a.item_off = item_off;
  a.tile_off = tile_off;
  a.tile_info = tile_info;
  a.items = items;
  a.part_o = part_o;
  a.part_lse = part_lse;
  a.O = static_cast<bf16_t*>(O);
  a.LSE = nullptr;
  a.L = pb.L;
  a.Lp = w.Lp;
  a.Lq = pb.Lq;
  a.q_pos0 = pb.q_pos0;
  a.Hq = pb.Hq;
  a.G = pb.G;
  a.S = 1024;  // only groups the window kernel's row tiles per XCD
  a.A = 1024;
  a.topk = pb.topk;
  a.n = n;
  a.window = window;
  a.ab = b;
  a.af = f;
  a.aroot = root;
  a.E = q.A;
  a.scale_log2e = pb.scale * kLog2e;
  a.qsh = pb.qsh;
  a.qst = pb.qst;
  a.kvsh = pb.kvsh;
  a.kvst = pb.kvst;

  const dim3 bgrid((unsigned)w.chunks, pb.Hq);
  hipLaunchKernelGGL(bucket_anchor_kernel<false>, bgrid, dim3(256), (size_t)n * sizeof(int), st, anchors,
                     blk_cnt, cursor, items, part_lse, pb.Lq, pb.q_pos0, pb.G, pb.topk, n, window, b, f, root,
                     a.E);
  hipLaunchKernelGGL(bucket_block_scan_kernel, dim3((n + 31) / 32, pb.Hkv), dim3(256), 0, st, blk_cnt, counts,
                     pb.G * w.chunks, n);
  hipLaunchKernelGGL(bucket_scan_kernel, dim3(1), dim3(1024), 0, st, counts, item_off, tile_off, cursor, w.B);
  hipLaunchKernelGGL(bucket_tiles_kernel, dim3(w.B), dim3(256), 0, st, tile_off, item_off, tile_info, items);
  hipLaunchKernelGGL(bucket_anchor_kernel<true>, bgrid, dim3(256), (size_t)4 * n * sizeof(int), st, anchors,
                     blk_cnt, cursor, items, part_lse, pb.Lq, pb.q_pos0, pb.G, pb.topk, n, window, b, f, root,
                     a.E);
  if (hipGetLastError() != hipSuccess) return SL_ERR_LAUNCH;
  if (pb.prof_start) (void)hipEventRecord(pb.prof_start, st);
  hipLaunchKernelGGL(span_flash_anchor_kernel, dim3(dev.grid), dim3(FlashLds<2>::kThreads),
                     FlashLds<2>::kBytes, st, a);
  if (pb.prof_stop) (void)hipEventRecord(pb.prof_stop, st);
  const unsigned lgrid = local_grid(pb.Lq, a.A, pb.Hkv, pb.G);
  hipLaunchKernelGGL(span_flash_local_kernel<false>, dim3(lgrid), dim3(FlashLds<1>::kThreads),
                     FlashLds<1>::kBytes, st, a);
  const int64_t rows = (int64_t)pb.Hq * pb.Lq;
  const dim3 mgrid((unsigned)((rows + 15) / 16));
  if (pb.topk <= 8)
    hipLaunchKernelGGL((merge_combined_kernel<8, true>), mgrid, dim3(256), 0, st, anchors, pb.gate, part_o,
                       part_lse, a.O, rows, pb.Lq, pb.q_pos0, 1, pb.topk);
  else if (pb.topk <= 16)
    hipLaunchKernelGGL((merge_combined_kernel<16, true>), mgrid, dim3(256), 0, st, anchors, pb.gate, part_o,
                       part_lse, a.O, rows, pb.Lq, pb.q_pos0, 1, pb.topk);
  else
    hipLaunchKernelGGL((merge_combined_kernel<32, true>), mgrid, dim3(256), 0, st, anchors, pb.gate, part_o,
                       part_lse, a.O, rows, pb.Lq, pb.q_pos0, 1, pb.topk);
  return hipGetLastError() == hipSuccess ? SL_OK : SL_ERR_LAUNCH;
}

}  // namespace sl
