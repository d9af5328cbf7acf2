// C-ABI layer: argument validation on the host, then dispatch to the kernel launchers.
// Nothing is enqueued before every check has passed.
#include <cmath>
#include <cstring>

#include "kernels.h"

namespace sl {

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Events armed by sl_set_profile_events for the calling thread's next operation.
thread_local hipEvent_t tl_prof_start = nullptr;
thread_local hipEvent_t tl_prof_stop = nullptr;

// Hands the armed events to a validated problem and disarms them.
void take_profile_events(Problem* pb) {
  pb->prof_start = tl_prof_start;
  pb->prof_stop = tl_prof_stop;
  tl_prof_start = tl_prof_stop = nullptr;
}

// Validates p for the given operation and fills pb.  Pure host code (no HIP call), so every
// error path can be exercised without a GPU.
sl_status make_problem(const sl_params* p, int op, Problem* pb) {
  if (!p) return SL_ERR_INVALID_ARG;
  if (p->L < 1 || p->Lq < 1 || p->q_pos0 < 0) return SL_ERR_INVALID_ARG;
  if (p->q_pos0 > p->L - p->Lq) return SL_ERR_INVALID_ARG;  // last query must be a visible key
  if (p->Hq < 1 || p->Hkv < 1 || p->Hq % p->Hkv != 0) return SL_ERR_INVALID_ARG;
  if (p->S < 1 || p->topk < 0) return SL_ERR_INVALID_ARG;
  if (p->span_stride < 0 || p->span_stride > p->S) return SL_ERR_INVALID_ARG;
  if (p->dtype != SL_F32 && p->dtype != SL_BF16) return SL_ERR_INVALID_ARG;
  if (!(p->scale >= 0.f) || std::isinf(p->scale)) return SL_ERR_INVALID_ARG;
  const bool is_search = (op == SL_OP_SEARCH_PREFILL || op == SL_OP_SEARCH_DECODE);
  const bool is_decode = (op == SL_OP_SEARCH_DECODE || op == SL_OP_ATTENTION_DECODE);
  if (op < SL_OP_SEARCH_PREFILL || op > SL_OP_ATTENTION_DECODE) return SL_ERR_INVALID_ARG;
  if (is_search && p->topk < 1) return SL_ERR_INVALID_ARG;
  if (is_decode && p->Lq != 1) return SL_ERR_INVALID_ARG;
  if (p->D != 64 && p->D != 128) return SL_ERR_UNSUPPORTED;
  if (p->topk > SL_MAX_TOPK) return SL_ERR_UNSUPPORTED;
  if (p->Hq / p->Hkv > 64) return SL_ERR_UNSUPPORTED;
  // Extents that keep every size and offset computed from them inside 64 bits: at most 2^40
  // tokens, token strides below 2^20 elements, head strides below 2^60.
  constexpr int64_t kMaxTokens = (int64_t)1 << 40, kMaxTokenStride = (int64_t)1 << 20,
                    kMaxHeadStride = (int64_t)1 << 60;
  if (p->L > kMaxTokens) return SL_ERR_UNSUPPORTED;
  if (p->Lq > (((int64_t)1 << 31) - 1) / p->Hq) return SL_ERR_UNSUPPORTED;  // row ids are 32-bit
  if (p->q_stride_t < 0 || p->kv_stride_t < 0 || p->q_stride_h < 0 || p->kv_stride_h < 0)
    return SL_ERR_INVALID_ARG;
  if (p->q_stride_t > kMaxTokenStride || p->kv_stride_t > kMaxTokenStride ||
      p->q_stride_h > kMaxHeadStride || p->kv_stride_h > kMaxHeadStride)
    return SL_ERR_UNSUPPORTED;

  const int64_t epl = p->dtype == SL_BF16 ? 8 : 4;  // elements per 16 bytes
  const int64_t qst = p->q_stride_t ? p->q_stride_t : p->D;
  const int64_t qsh = p->q_stride_h ? p->q_stride_h : p->Lq * qst;
  const int64_t kvst = p->kv_stride_t ? p->kv_stride_t : p->D;
  const int64_t kvsh = p->kv_stride_h ? p->kv_stride_h : p->L * kvst;
  if (qst < p->D || kvst < p->D) return SL_ERR_INVALID_ARG;
  if (qst % epl || qsh % epl || kvst % epl || kvsh % epl) return SL_ERR_INVALID_ARG;

  pb->L = p->L;
  pb->Lq = p->Lq;
  pb->q_pos0 = p->q_pos0;
  pb->Hq = p->Hq;
  pb->Hkv = p->Hkv;
  pb->G = p->Hq / p->Hkv;
  pb->D = p->D;
  pb->S = p->S;
  pb->A = p->span_stride ? p->span_stride : p->S;
  pb->topk = p->topk;
  pb->dtype = p->dtype;
  pb->scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->D);
  pb->qsh = qsh;
  pb->qst = qst;
  pb->kvsh = kvsh;
  pb->kvsh_given = p->kv_stride_h != 0;
  pb->kvst = kvst;
  pb->n = (p->L + pb->A - 1) / pb->A;
  pb->prof_start = nullptr;
  pb->prof_stop = nullptr;
  pb->combined = false;
  pb->gate = nullptr;
  return SL_OK;
}

size_t ws_bytes_for(const Problem& pb, int op) {
  switch (op) {
    case SL_OP_SEARCH_PREFILL: return prefill_search_ws_bytes(pb);
    case SL_OP_SEARCH_DECODE: return decode_search_ws_bytes(pb);
    case SL_OP_ATTENTION_PREFILL: return prefill_attention_ws_bytes(pb);
    case SL_OP_ATTENTION_DECODE: return decode_attention_ws_bytes(pb);
  }
  return 0;
}

sl_status check_ws(const Problem& pb, int op, const void* ws, size_t ws_bytes) {
  const size_t need = ws_bytes_for(pb, op);
  if (need == 0) return SL_OK;
  if (!ws || ws_bytes < need) return SL_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return SL_ERR_WORKSPACE;
  return SL_OK;
}

sl_status search_entry(const sl_params* p, int op, const void* Qs, const void* K, const void* Ks,
                       int32_t* idx, float* scores, void* ws, size_t ws_bytes, void* stream) {
  Problem pb;
  sl_status s = make_problem(p, op, &pb);
  if (s != SL_OK) return s;
  if (!Qs || !idx || (!K && !Ks)) return SL_ERR_INVALID_ARG;
  if (!aligned16(Qs) || !aligned16(K) || !aligned16(Ks) || !aligned16(idx) || !aligned16(scores))
    return SL_ERR_INVALID_ARG;
  s = check_ws(pb, op, ws, ws_bytes);
  if (s != SL_OK) return s;
  take_profile_events(&pb);
  pb.S = pb.A;  // span-search only sees the anchor grid
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (op == SL_OP_SEARCH_DECODE) return decode_search(pb, Qs, K, Ks, idx, scores, ws, st);
  return prefill_search(pb, Qs, K, Ks, idx, scores, ws, st);
}

// `combined`: the gated form (scores required when topk > 0, no LSE); otherwise LSE is required.
sl_status attention_entry(const sl_params* p, int op, const void* Q, const void* K, const void* V,
                          const int32_t* idx, const float* scores, bool combined, void* O,
                          float* LSE, void* ws, size_t ws_bytes, void* stream) {
  Problem pb;
  sl_status s = make_problem(p, op, &pb);
  if (s != SL_OK) return s;
  if (!Q || !K || !V || !O || (!combined && !LSE)) return SL_ERR_INVALID_ARG;
  if (pb.topk > 0 && (!idx || (combined && !scores))) return SL_ERR_INVALID_ARG;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(idx) ||
      !aligned16(LSE) || !aligned16(scores))
    return SL_ERR_INVALID_ARG;
  pb.combined = combined;
  pb.gate = scores;
  s = check_ws(pb, op, ws, ws_bytes);
  if (s != SL_OK) return s;
  take_profile_events(&pb);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (op == SL_OP_ATTENTION_DECODE) return decode_attention(pb, Q, K, V, idx, O, LSE, ws, st);
  return prefill_attention(pb, Q, K, V, idx, O, LSE, ws, st);
}

}  // namespace

}  // namespace sl

extern "C" {

size_t sl_workspace_bytes(const sl_params* p, int op) {
  sl::Problem pb;
  if (sl::make_problem(p, op, &pb) != SL_OK) return SL_WORKSPACE_INVALID;
  return sl::ws_bytes_for(pb, op);
}

void sl_set_profile_events(void* start, void* stop) {
  const bool both = start && stop;
  sl::tl_prof_start = both ? static_cast<hipEvent_t>(start) : nullptr;
  sl::tl_prof_stop = both ? static_cast<hipEvent_t>(stop) : nullptr;
}

sl_status sl_span_keys(const sl_params* p, const void* K, void* Ks, void* hip_stream) {
  if (!p) return SL_ERR_INVALID_ARG;
  sl_params q = *p;  // only L, Hkv, D, S, dtype and the kv strides matter here
  q.Lq = 1;
  q.q_pos0 = 0;
  q.Hq = q.Hkv;
  q.topk = 0;
  q.scale = 0.f;
  q.q_stride_h = q.q_stride_t = 0;
  sl::Problem pb;
  sl_status s = sl::make_problem(&q, SL_OP_ATTENTION_PREFILL, &pb);
  if (s != SL_OK) return s;
  if (!K || !Ks || !sl::aligned16(K) || !sl::aligned16(Ks)) return SL_ERR_INVALID_ARG;
  pb.S = pb.A;  // keys sit on the anchor grid
  return sl::span_keys(pb, K, Ks, static_cast<hipStream_t>(hip_stream));
}

sl_status sl_span_search_prefill(const sl_params* p, const void* Qs, const void* K, const void* Ks,
                                 int32_t* idx, float* scores, void* ws, size_t ws_bytes,
                                 void* hip_stream) {
  return sl::search_entry(p, SL_OP_SEARCH_PREFILL, Qs, K, Ks, idx, scores, ws, ws_bytes, hip_stream);
}

sl_status sl_span_search_decode(const sl_params* p, const void* Qs, const void* K, const void* Ks,
                                int32_t* idx, float* scores, void* ws, size_t ws_bytes,
                                void* hip_stream) {
  return sl::search_entry(p, SL_OP_SEARCH_DECODE, Qs, K, Ks, idx, scores, ws, ws_bytes, hip_stream);
}

sl_status sl_span_attention_prefill(const sl_params* p, const void* Q, const void* K, const void* V,
                                    const int32_t* idx, void* O, float* LSE, void* ws,
                                    size_t ws_bytes, void* hip_stream) {
  return sl::attention_entry(p, SL_OP_ATTENTION_PREFILL, Q, K, V, idx, nullptr, false, O, LSE, ws,
                             ws_bytes, hip_stream);
}

sl_status sl_span_attention_decode(const sl_params* p, const void* Q, const void* K, const void* V,
                                   const int32_t* idx, void* O, float* LSE, void* ws,
                                   size_t ws_bytes, void* hip_stream) {
  return sl::attention_entry(p, SL_OP_ATTENTION_DECODE, Q, K, V, idx, nullptr, false, O, LSE, ws,
                             ws_bytes, hip_stream);
}

size_t sl_noalloc_scratch_bytes(void) { return sl::decode_attention_static_scratch_bytes(); }

sl_status sl_span_attention_decode_noalloc(const sl_params* p, const void* Q, const void* K,
                                           const void* V, const int32_t* idx, void* O, float* LSE,
                                           void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb);
  if (s != SL_OK) return s;
  if (!Q || !K || !V || !O || !LSE || (pb.topk > 0 && !idx)) return SL_ERR_INVALID_ARG;
  if (!sl::aligned16(Q) || !sl::aligned16(K) || !sl::aligned16(V) || !sl::aligned16(O) ||
      !sl::aligned16(idx) || !sl::aligned16(LSE))
    return SL_ERR_INVALID_ARG;
  return sl::decode_attention_static(pb, Q, K, V, idx, O, LSE, static_cast<hipStream_t>(hip_stream));
}

sl_status sl_span_attention_combined_prefill(const sl_params* p, const void* Q, const void* K,
                                             const void* V, const int32_t* idx, const float* scores,
                                             void* O, void* ws, size_t ws_bytes, void* hip_stream) {
  return sl::attention_entry(p, SL_OP_ATTENTION_PREFILL, Q, K, V, idx, scores, true, O, nullptr, ws,
                             ws_bytes, hip_stream);
}

sl_status sl_span_attention_combined_decode(const sl_params* p, const void* Q, const void* K,
                                            const void* V, const int32_t* idx, const float* scores,
                                            void* O, void* ws, size_t ws_bytes, void* hip_stream) {
  return sl::attention_entry(p, SL_OP_ATTENTION_DECODE, Q, K, V, idx, scores, true, O, nullptr, ws,
                             ws_bytes, hip_stream);
}

// 0 if the geometry is invalid, else the root 1/p (2 or 3; search_root = 0 means 2)
static int anchor_root(const sl_anchor_geometry* g) {
  if (!g || g->window < 0 || g->backward_factor < 0 || g->forward_factor < 0) return 0;
  if (g->search_root == 0 || g->search_root == 2) return 2;
  return g->search_root == 3 ? 3 : 0;
}

size_t sl_anchor_workspace_bytes(const sl_params* p, const sl_anchor_geometry* g) {
  sl::Problem pb;
  const int root = anchor_root(g);
  if (!root) return SL_WORKSPACE_INVALID;
  if (sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb) != SL_OK) return SL_WORKSPACE_INVALID;
  return sl::anchor_attention_ws_bytes(pb, g->window, g->backward_factor, g->forward_factor, root);
}

sl_status sl_anchor_search_decode(const sl_params* p, const sl_anchor_geometry* g, const void* Qs,
                                  const void* K, int32_t* anchors, float* scores, void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_SEARCH_DECODE, &pb);
  if (s != SL_OK) return s;
  const int root = anchor_root(g);
  if (!root || !Qs || !K || !anchors) return SL_ERR_INVALID_ARG;
  if (!sl::aligned16(Qs) || !sl::aligned16(K) || !sl::aligned16(anchors) || !sl::aligned16(scores))
    return SL_ERR_INVALID_ARG;
  if (pb.L > ((int64_t)1 << 31) - 1) return SL_ERR_UNSUPPORTED;  // anchors are int32 token positions
  sl::take_profile_events(&pb);
  return sl::anchor_search_decode(pb, g->window, root, Qs, K, anchors, scores,
                                  static_cast<hipStream_t>(hip_stream));
}

sl_status sl_anchor_attention_decode(const sl_params* p, const sl_anchor_geometry* g, const void* Q,
                                     const void* K, const void* V, const int32_t* anchors,
                                     const float* scores, void* O, void* ws, size_t ws_bytes,
                                     void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb);
  if (s != SL_OK) return s;
  const int root = anchor_root(g);
  if (!root) return SL_ERR_INVALID_ARG;
  if (!Q || !K || !V || !O || (pb.topk > 0 && (!anchors || !scores))) return SL_ERR_INVALID_ARG;
  if (!sl::aligned16(Q) || !sl::aligned16(K) || !sl::aligned16(V) || !sl::aligned16(O) ||
      !sl::aligned16(anchors) || !sl::aligned16(scores))
    return SL_ERR_INVALID_ARG;
  if (pb.L > ((int64_t)1 << 31) - 1) return SL_ERR_UNSUPPORTED;
  const size_t need = sl::anchor_attention_ws_bytes(pb, g->window, g->backward_factor, g->forward_factor, root);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SL_ERR_WORKSPACE;
  pb.combined = true;
  pb.gate = scores;
  sl::take_profile_events(&pb);
  return sl::anchor_attention_decode(pb, g->window, g->backward_factor, g->forward_factor, root, Q, K,
                                     V, anchors, O, ws, static_cast<hipStream_t>(hip_stream));
}

sl_status sl_anchor_search_prefill(const sl_params* p, const sl_anchor_geometry* g, const void* Qs,
                                   const void* K, int32_t* anchors, float* scores, void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_SEARCH_PREFILL, &pb);
  if (s != SL_OK) return s;
  const int root = anchor_root(g);
  if (!root || !Qs || !K || !anchors) return SL_ERR_INVALID_ARG;
  if (!sl::aligned16(Qs) || !sl::aligned16(K) || !sl::aligned16(anchors) || !sl::aligned16(scores))
    return SL_ERR_INVALID_ARG;
  if (pb.L > ((int64_t)1 << 31) - 1) return SL_ERR_UNSUPPORTED;  // anchors are int32 token positions
  sl::take_profile_events(&pb);
  return sl::anchor_search_prefill(pb, g->window, root, Qs, K, anchors, scores,
                                   static_cast<hipStream_t>(hip_stream));
}

size_t sl_anchor_prefill_workspace_bytes(const sl_params* p, const sl_anchor_geometry* g) {
  sl::Problem pb;
  const int root = anchor_root(g);
  if (!root) return SL_WORKSPACE_INVALID;
  if (sl::make_problem(p, SL_OP_ATTENTION_PREFILL, &pb) != SL_OK) return SL_WORKSPACE_INVALID;
  return sl::prefill_anchor_mfma_supported(pb, g->window) ? sl::prefill_anchor_mfma_ws_bytes(pb) : 0;
}

sl_status sl_anchor_attention_prefill(const sl_params* p, const sl_anchor_geometry* g, const void* Q,
                                      const void* K, const void* V, const int32_t* anchors,
                                      const float* scores, void* O, void* ws, size_t ws_bytes,
                                      void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_ATTENTION_PREFILL, &pb);
  if (s != SL_OK) return s;
  const int root = anchor_root(g);
  if (!root) return SL_ERR_INVALID_ARG;
  if (!Q || !K || !V || !O || (pb.topk > 0 && (!anchors || !scores))) return SL_ERR_INVALID_ARG;
  if (!sl::aligned16(Q) || !sl::aligned16(K) || !sl::aligned16(V) || !sl::aligned16(O) ||
      !sl::aligned16(anchors) || !sl::aligned16(scores))
    return SL_ERR_INVALID_ARG;
  if (pb.L > ((int64_t)1 << 31) - 1) return SL_ERR_UNSUPPORTED;
  pb.combined = true;
  pb.gate = scores;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // the matrix-core form needs scratch; without one (ws == NULL) the row-stationary kernels run
  if (ws && sl::prefill_anchor_mfma_supported(pb, g->window)) {
    if (ws_bytes < sl::prefill_anchor_mfma_ws_bytes(pb) || (reinterpret_cast<uintptr_t>(ws) & 255u))
      return SL_ERR_WORKSPACE;
    sl::take_profile_events(&pb);
    return sl::prefill_anchor_attention_mfma(pb, g->window, g->backward_factor, g->forward_factor, root, Q, K, V,
                                             anchors, O, ws, st);
  }
  sl::take_profile_events(&pb);
  return sl::anchor_attention_prefill(pb, g->window, g->backward_factor, g->forward_factor, root, Q, K,
                                      V, anchors, O, st);
}

size_t sl_decode_batched_workspace_bytes(const sl_params* p, int32_t B) {
  sl::Problem pb;
  if (B < 1 || sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb) != SL_OK) return SL_WORKSPACE_INVALID;
  return sl::decode_attention_batched_ws_bytes(pb, B);
}

sl_status sl_span_search_decode_batched(const sl_params* p, const sl_decode_seq* seqs, int32_t B,
                                        void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_SEARCH_DECODE, &pb);
  if (s != SL_OK) return s;
  if (!seqs || B < 1 || B > 65535 || (reinterpret_cast<uintptr_t>(seqs) & 7u)) return SL_ERR_INVALID_ARG;
  pb.S = pb.A;  // span-search only sees the anchor grid
  return sl::decode_search_batched(pb, seqs, B, static_cast<hipStream_t>(hip_stream));
}

sl_status sl_span_attention_decode_batched(const sl_params* p, const sl_decode_seq* seqs, int32_t B,
                                           void* ws, size_t ws_bytes, void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb);
  if (s != SL_OK) return s;
  if (!seqs || B < 1 || B > 65535 || (reinterpret_cast<uintptr_t>(seqs) & 7u)) return SL_ERR_INVALID_ARG;
  const size_t need = sl::decode_attention_batched_ws_bytes(pb, B);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SL_ERR_WORKSPACE;
  return sl::decode_attention_batched(pb, seqs, B, ws, static_cast<hipStream_t>(hip_stream));
}

static bool good_batch(const sl_decode_seq* seqs, int32_t B) {
  return seqs && B >= 1 && B <= 65535 && (reinterpret_cast<uintptr_t>(seqs) & 7u) == 0;
}

sl_status sl_span_attention_combined_decode_batched(const sl_params* p, const sl_decode_seq* seqs,
                                                    int32_t B, void* ws, size_t ws_bytes,
                                                    void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb);
  if (s != SL_OK) return s;
  if (!good_batch(seqs, B)) return SL_ERR_INVALID_ARG;
  const size_t need = sl::decode_attention_batched_ws_bytes(pb, B);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SL_ERR_WORKSPACE;
  pb.combined = true;
  return sl::decode_attention_batched(pb, seqs, B, ws, static_cast<hipStream_t>(hip_stream));
}

size_t sl_anchor_batched_workspace_bytes(const sl_params* p, const sl_anchor_geometry* g, int32_t B) {
  sl::Problem pb;
  const int root = anchor_root(g);
  if (!root || B < 1) return SL_WORKSPACE_INVALID;
  if (sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb) != SL_OK) return SL_WORKSPACE_INVALID;
  return sl::anchor_attention_batched_ws_bytes(pb, g->window, g->backward_factor, g->forward_factor, root, B);
}

sl_status sl_anchor_search_decode_batched(const sl_params* p, const sl_anchor_geometry* g,
                                          const sl_decode_seq* seqs, int32_t B, void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_SEARCH_DECODE, &pb);
  if (s != SL_OK) return s;
  const int root = anchor_root(g);
  if (!root || !good_batch(seqs, B)) return SL_ERR_INVALID_ARG;
  if (pb.L > ((int64_t)1 << 31) - 1) return SL_ERR_UNSUPPORTED;  // anchors are int32 token positions
  return sl::anchor_search_decode_batched(pb, g->window, root, seqs, B, static_cast<hipStream_t>(hip_stream));
}

sl_status sl_anchor_attention_decode_batched(const sl_params* p, const sl_anchor_geometry* g,
                                             const sl_decode_seq* seqs, int32_t B, void* ws,
                                             size_t ws_bytes, void* hip_stream) {
  sl::Problem pb;
  sl_status s = sl::make_problem(p, SL_OP_ATTENTION_DECODE, &pb);
  if (s != SL_OK) return s;
  const int root = anchor_root(g);
  if (!root || !good_batch(seqs, B)) return SL_ERR_INVALID_ARG;
  if (pb.L > ((int64_t)1 << 31) - 1) return SL_ERR_UNSUPPORTED;
  const size_t need =
      sl::anchor_attention_batched_ws_bytes(pb, g->window, g->backward_factor, g->forward_factor, root, B);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SL_ERR_WORKSPACE;
  pb.combined = true;
  return sl::anchor_attention_decode_batched(pb, g->window, g->backward_factor, g->forward_factor, root,
                                             seqs, B, ws, static_cast<hipStream_t>(hip_stream));
}

const char* sl_status_string(sl_status status) {
  switch (status) {
    case SL_OK: return "SL_OK";
    case SL_ERR_INVALID_ARG: return "SL_ERR_INVALID_ARG: bad pointer, size, stride or alignment";
    case SL_ERR_UNSUPPORTED: return "SL_ERR_UNSUPPORTED: outside the compiled envelope (D, topk, dtype, span count)";
    case SL_ERR_WORKSPACE: return "SL_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case SL_ERR_LAUNCH: return "SL_ERR_LAUNCH: HIP failed to enqueue a kernel";
  }
  return "unknown sl_status";
}

int sl_version(void) { return 400; }  // 0.4.0: sl_anchor_attention_prefill takes a workspace (matrix-core form)

}  // extern "C"
