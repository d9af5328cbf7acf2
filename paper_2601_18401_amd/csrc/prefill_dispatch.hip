// Chooses the prefill implementation for a problem: the matrix-core path where it applies,
// otherwise the row-stationary kernels.
#include "kernels.h"

namespace sl {

size_t prefill_search_ws_bytes(const Problem&) { return 0; }

sl_status prefill_search(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                         int32_t* idx, float* scores, void* /*ws*/, hipStream_t st) {
  if (prefill_search_mfma_supported(pb)) return prefill_search_mfma(pb, Qs, K, Ks, idx, scores, st);
  return prefill_search_rows(pb, Qs, K, Ks, idx, scores, st);
}

size_t prefill_attention_ws_bytes(const Problem& pb) {
  return prefill_attention_mfma_supported(pb) ? prefill_attention_mfma_ws_bytes(pb) : 0;
}

sl_status prefill_attention(const Problem& pb, const void* Q, const void* K, const void* V,
                            const int32_t* idx, void* O, float* LSE, void* ws, hipStream_t st) {
  if (prefill_attention_mfma_supported(pb))
    return prefill_attention_mfma(pb, Q, K, V, idx, O, LSE, ws, st);
  return prefill_attention_rows(pb, Q, K, V, idx, O, LSE, st);
}

}  // namespace sl
