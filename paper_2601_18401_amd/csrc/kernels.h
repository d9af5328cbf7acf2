// Internal launch interface between the C-ABI layer (api.hip) and the kernel translation units.
#pragma once

#include "sl_common.h"

namespace sl {

// a0: span-key gather
sl_status span_keys(const Problem& pb, const void* K, void* Ks, hipStream_t st);

// a7: decode span-search (score kernel + select kernel)
size_t decode_search_ws_bytes(const Problem& pb);
sl_status decode_search(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                        int32_t* idx, float* scores, void* ws, hipStream_t st);

// a8 + a9: decode span-attention (split-KV + reduce)
size_t decode_attention_ws_bytes(const Problem& pb);
sl_status decode_attention(const Problem& pb, const void* Q, const void* K, const void* V,
                           const int32_t* idx, void* O, float* LSE, void* ws, hipStream_t st);

// a8 + a9 with the partial records in a device array of the library (no workspace argument)
size_t decode_attention_static_scratch_bytes();
sl_status decode_attention_static(const Problem& pb, const void* Q, const void* K, const void* V,
                                  const int32_t* idx, void* O, float* LSE, hipStream_t st);

// a7 .. a9 for a batch of sequences (one more grid dimension; tensors and lengths per sequence
// come from a device array)
sl_status decode_search_batched(const Problem& pb, const sl_decode_seq* seqs, int B, hipStream_t st);
size_t decode_attention_batched_ws_bytes(const Problem& pb, int B);
sl_status decode_attention_batched(const Problem& pb, const sl_decode_seq* seqs, int B, void* ws,
                                   hipStream_t st);

// ... and on the paper's own geometry (anchors as candidates, gated combination)
sl_status anchor_search_decode_batched(const Problem& pb, int64_t window, int root,
                                       const sl_decode_seq* seqs, int B, hipStream_t st);
size_t anchor_attention_batched_ws_bytes(const Problem& pb, int64_t window, int b, int f, int root, int B);
sl_status anchor_attention_decode_batched(const Problem& pb, int64_t window, int b, int f, int root,
                                          const sl_decode_seq* seqs, int B, void* ws, hipStream_t st);

// The paper's own geometry, decode form (Section 3.3, Algorithm 1): anchors on the quadratic
// stride pattern, spans of b*l(i) / f*l(i) tokens around the selected anchors, window w.
// root = 1/p: 2 (anchors i-(s+1)^2+1, l = ceil(sqrt(i))) or 3 (anchors i-(s+1)^3+1, l = ceil(i^(2/3))).
sl_status anchor_search_decode(const Problem& pb, int64_t window, int root, const void* Qs,
                               const void* K, int32_t* anchors, float* scores, hipStream_t st);
size_t anchor_attention_ws_bytes(const Problem& pb, int64_t window, int b, int f, int root);
sl_status anchor_attention_decode(const Problem& pb, int64_t window, int b, int f, int root,
                                  const void* Q, const void* K, const void* V,
                                  const int32_t* anchors, void* O, void* ws, hipStream_t st);

// The same geometry, prefill form (one wavefront per query row; every row has its own anchors,
// span length and window)
sl_status anchor_search_prefill(const Problem& pb, int64_t window, int root, const void* Qs,
                                const void* K, int32_t* anchors, float* scores, hipStream_t st);
sl_status anchor_attention_prefill(const Problem& pb, int64_t window, int b, int f, int root,
                                   const void* Q, const void* K, const void* V,
                                   const int32_t* anchors, void* O, hipStream_t st);

// ... and its span-attention + combination on the matrix cores (bf16, D = 128, window >= 1)
bool prefill_anchor_mfma_supported(const Problem& pb, int64_t window);
size_t prefill_anchor_mfma_ws_bytes(const Problem& pb);
sl_status prefill_anchor_attention_mfma(const Problem& pb, int64_t window, int b, int f, int root,
                                        const void* Q, const void* K, const void* V,
                                        const int32_t* anchors, void* O, void* ws, hipStream_t st);

// a1 + a2: prefill span-search
size_t prefill_search_ws_bytes(const Problem& pb);
sl_status prefill_search(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                         int32_t* idx, float* scores, void* ws, hipStream_t st);

// a1 + a2, row-stationary form (fp32 and shapes outside the matrix-core path)
sl_status prefill_search_rows(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                              int32_t* idx, float* scores, hipStream_t st);

// a4 .. a6, row-stationary form
sl_status prefill_attention_rows(const Problem& pb, const void* Q, const void* K, const void* V,
                                 const int32_t* idx, void* O, float* LSE, hipStream_t st);

// a1 + a2 on the matrix cores (bf16, D = 128)
bool prefill_search_mfma_supported(const Problem& pb);
sl_status prefill_search_mfma(const Problem& pb, const void* Qs, const void* K, const void* Ks,
                              int32_t* idx, float* scores, hipStream_t st);

// a3 .. a6 on the matrix cores (bf16, D = 128, S % 64 == 0)
bool prefill_attention_mfma_supported(const Problem& pb);
size_t prefill_attention_mfma_ws_bytes(const Problem& pb);
sl_status prefill_attention_mfma(const Problem& pb, const void* Q, const void* K, const void* V,
                                 const int32_t* idx, void* O, float* LSE, void* ws, hipStream_t st);

// a3 .. a6: prefill span-attention
size_t prefill_attention_ws_bytes(const Problem& pb);
sl_status prefill_attention(const Problem& pb, const void* Q, const void* K, const void* V,
                            const int32_t* idx, void* O, float* LSE, void* ws, hipStream_t st);

}  // namespace sl
