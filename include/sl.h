/* sl.h -- C ABI of the Superlinear attention (N = 2) span-search / span-attention library
 * for AMD MI355X (gfx950).
 *
 * The library implements the two data-parallel steps of the baseline N = 2 instantiation of
 * Superlinear multi-step attention on a fixed span grid:
 *
 *   span-search    (paper Section 3.2, eq. (2) and (3); Algorithm 1, the scoring loop and TopK):
 *                  score every candidate span of a causal query by the raw dot product of the
 *                  search query with the span's search key, keep the top-k spans.
 *   span-attention (paper Section 3.3, eq. (4); Algorithm 1, the DedupConcat + Attention steps
 *                  and the empty-selection branch): exact softmax attention of the query over
 *                  the union of the selected spans and its local window; returns the output
 *                  and the log-sum-exp of the logits.
 *   combination    (paper Section 3.4, eq. (5) and (6); Algorithm 1's last two steps), as a
 *                  second form of span-attention: one softmax per selected span (merged with
 *                  the local window), gated by the softmax of the selected search scores.
 *
 * Geometry.  Tokens 0 .. L-1; span j is the token range [j*S, min((j+1)*S, L) - 1]; its anchor
 * (search position) is its last token (j+1)*S - 1 (Algorithm 1's span [t - b*l, t + f*l] with
 * f = 0, b*l = S).  Query row r has absolute position i = q_pos0 + r and lies in span
 * c = i / S.  Its candidates are the complete spans j < c (Algorithm 1 removes the window's
 * indices from the anchor candidates); its local window is [c*S, i].  (sl_params.span_stride
 * turns this into a grid of overlapping spans.)
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never allocates,
 *     frees or synchronises.  Work is enqueued on `hip_stream` (a hipStream_t, NULL = the
 *     default stream) and completes asynchronously.
 *   - Layouts (element strides, innermost dimension D contiguous):
 *       Q, Qs, O : [Hq ][Lq][D]  strides (q_stride_h, q_stride_t, 1);  O is always packed [Hq][Lq][D]
 *       K, V     : [Hkv][L ][D]  strides (kv_stride_h, kv_stride_t, 1)
 *       Ks       : [Hkv][n ][D]  packed, n = ceil(L / S); row j = search key of span j
 *       idx      : [Hq ][Lq][topk] int32, packed
 *       scores   : [Hq ][Lq][topk] float, packed
 *       LSE      : [Hq ][Lq] float, packed
 *     A stride given as 0 means "packed".  Query head h reads KV head h / (Hq / Hkv).
 *   - dtype selects the element type of Q, Qs, K, V, Ks and O (fp32, or bf16 with fp32
 *     accumulation); scores, LSE and all softmax statistics are fp32.
 *   - Base pointers must be 16-byte aligned and strides multiples of 16 bytes.
 *   - Errors: every argument is validated on the host before anything is enqueued; on error
 *     nothing has been launched and a status other than SL_OK is returned (no exceptions, no
 *     abort).  A failed kernel launch returns SL_ERR_LAUNCH.
 *   - Scratch memory comes from the caller through (ws, ws_bytes); ask sl_workspace_bytes for
 *     the size.  ws must be 256-byte aligned.  Calls that share a workspace must be ordered on
 *     one stream.
 */
#ifndef SL_H_
#define SL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SL_OK = 0,
  SL_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad stride or alignment, ...     */
  SL_ERR_UNSUPPORTED = 2, /* valid request outside the compiled envelope (D, topk, dtype)      */
  SL_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or smaller than sl_workspace_bytes  */
  SL_ERR_LAUNCH = 4       /* HIP reported an error when enqueueing                             */
} sl_status;

typedef enum { SL_F32 = 0, SL_BF16 = 1 } sl_dtype;

typedef enum {
  SL_OP_SEARCH_PREFILL = 0,
  SL_OP_SEARCH_DECODE = 1,
  SL_OP_ATTENTION_PREFILL = 2,
  SL_OP_ATTENTION_DECODE = 3
} sl_op;

/* Largest supported top-k (routed spans per query and head; the local window is extra). */
#define SL_MAX_TOPK 32

typedef struct sl_params {
  int64_t L;       /* keys visible: sequence length (prefill) or cache length incl. the current token (decode) */
  int64_t Lq;      /* query rows per head; decode entry points require Lq == 1                    */
  int64_t q_pos0;  /* absolute position of query row 0 (prefill: 0, or chunk start; decode: L-1)   */
  int32_t Hq;      /* query heads                                                                  */
  int32_t Hkv;     /* key/value heads, Hq % Hkv == 0                                               */
  int32_t D;       /* head dimension: 64 or 128                                                    */
  int32_t S;       /* span length in tokens, >= 1                                                  */
  int32_t topk;    /* routed spans per (head, query): 1..SL_MAX_TOPK for search, 0..SL_MAX_TOPK for attention */
  int32_t dtype;   /* sl_dtype                                                                     */
  float scale;     /* softmax scale of span-attention; 0 means 1/sqrt(D). Search scores are unscaled (eq. (2)) */
  int32_t span_stride; /* anchor spacing A in tokens: 0 (or S) = the disjoint grid described above.
                          0 < A < S is the redundant grid (Section 2.4, p_sh + p_sp > 1; Section 4.4's
                          redundancy factors): anchors at (j+1)*A - 1, span j = the S tokens ending at its
                          anchor, [max(0, (j+1)*A - S), (j+1)*A - 1], so neighbouring spans overlap;
                          c = i / A, candidates j < c, window [c*A, i]; span-attention's joint softmax
                          runs over the UNION of the selected spans and the window (every token once).
                          Span-search and sl_span_keys only see the anchor grid: they use A where the
                          text says S. */
  int64_t q_stride_h, q_stride_t;   /* element strides of Q / Qs; 0 = packed                       */
  int64_t kv_stride_h, kv_stride_t; /* element strides of K and V; 0 = packed                      */
} sl_params;

/* Returned by the *_workspace_bytes functions for parameters the entry point would reject. */
#define SL_WORKSPACE_INVALID ((size_t)-1)

/* Bytes of scratch the given operation needs for these parameters: 0 if it needs none,
 * SL_WORKSPACE_INVALID if the parameters are invalid or unsupported (the entry point itself
 * reports why). Host-only, no HIP call. */
size_t sl_workspace_bytes(const sl_params* p, int op /* sl_op */);

/* Optional profiling hook (benchmarks; no part of the operations).  Arms two caller-owned
 * hipEvent_t handles for the NEXT span-search or span-attention call made by the calling thread
 * (single-sequence entry points): that call records `start` immediately before, and `stop`
 * immediately after, its dominant kernel (the K/V-streaming kernel of span-attention, the scoring
 * kernel of span-search; the decode span-attention entry point attaches them to that kernel's
 * dispatch, so that they hold the kernel's own begin and end timestamps), and disarms them.
 * Passing NULL for either disarms.  Do not arm while the stream is capturing. */
void sl_set_profile_events(void* start, void* stop);

/* Span-key formation.  Section 3.5 / 4.2: the representative stream reuses the key tensor,
 * K_a = K, so the search key of span j is K at the span's anchor.  Gathers
 * Ks[kv][j][:] = K[kv][(j+1)*S - 1][:] for every complete span j < L / S into the packed
 * tensor Ks [Hkv][ceil(L/S)][D] (device memory, caller-owned; the row of a trailing partial
 * span is left untouched).  Uses L, Hkv, D, S, dtype and the kv strides of p. */
sl_status sl_span_keys(const sl_params* p, const void* K, void* Ks, void* hip_stream);

/* Span-search, prefill form (Section 3.2, eq. (2)-(3); Algorithm 1 scoring loop + TopK) for
 * Lq query rows per head at positions q_pos0 .. q_pos0 + Lq - 1.
 *   Qs     search queries Q_s, layout of Q.
 *   K      key tensor; only read when Ks == NULL (then span j's key is K[kv][(j+1)*S-1]).
 *   Ks     packed span search keys, or NULL.
 *   idx    out: for each (h, r) the min(topk, c) best candidate spans in ASCENDING span index,
 *          remaining slots -1.  Ties in score go to the lower span index.
 *   scores out, optional (NULL to skip): fp32 score of the span in the same slot, -inf in
 *          empty slots.
 * Scores are accumulated in fp32 from exact products of the inputs. */
sl_status sl_span_search_prefill(const sl_params* p, const void* Qs, const void* K, const void* Ks,
                                 int32_t* idx, float* scores, void* ws, size_t ws_bytes,
                                 void* hip_stream);

/* Span-search, decode form: the same operation for one query row per head (Lq must be 1) at
 * position q_pos0 against an L-token cache (Section 4.3, decoding path: routing scores over
 * the anchor set of the current position).  Same arguments and outputs as the prefill form. */
sl_status sl_span_search_decode(const sl_params* p, const void* Qs, const void* K, const void* Ks,
                                int32_t* idx, float* scores, void* ws, size_t ws_bytes,
                                void* hip_stream);

/* Span-attention, prefill form (Section 3.3, eq. (4); Algorithm 1 DedupConcat + Attention, and
 * the window-only branch when nothing is selected).  For each (h, r): one softmax over
 * J = union of spans idx[h][r][*] and the local window [c*S, i], logits scale * <Q, K_t>.
 *   idx    in: span indices as produced by span-search.  Entries < 0 or >= c are empty slots
 *          (so arbitrary garbage cannot cause an out-of-range read).  A row must not list a
 *          span twice: the result for such a row is unspecified (still memory-safe).  Distinct
 *          spans that overlap (span_stride < S) are de-duplicated: a token counts once.
 *   O      out: [Hq][Lq][D] in the input dtype.
 *   LSE    out: natural-log sum over J of exp(logit), fp32. */
sl_status sl_span_attention_prefill(const sl_params* p, const void* Q, const void* K, const void* V,
                                    const int32_t* idx, void* O, float* LSE, void* ws,
                                    size_t ws_bytes, void* hip_stream);

/* Span-attention, decode form: one query row per head (Lq must be 1) against an L-token KV
 * cache; split over the selected spans and merged by log-sum-exp (Section 4.3, decoding path:
 * attention over the routed spans, O(L^{1/2}) keys per step).  Same arguments as the prefill form. */
sl_status sl_span_attention_decode(const sl_params* p, const void* Q, const void* K, const void* V,
                                   const int32_t* idx, void* O, float* LSE, void* ws,
                                   size_t ws_bytes, void* hip_stream);

/* sl_span_attention_decode for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments, outputs and kernels as sl_span_attention_decode, but the split-KV partial
 * records live in a device array inside the library (sl_noalloc_scratch_bytes() bytes, 8 MiB, held
 * by every GPU the library runs on until the process ends) instead of (ws, ws_bytes).  The call
 * allocates and frees nothing.
 *   - The device that owns hip_stream must be the current device.  The array's address on a
 *     device is looked up on the first call there (not a stream operation).
 *   - A request whose records need more than the array (sl_workspace_bytes(p, SL_OP_ATTENTION_DECODE)
 *     > sl_noalloc_scratch_bytes()) returns SL_ERR_UNSUPPORTED and enqueues nothing.
 *   - All calls on one GPU share that GPU's array: calls that may overlap on a GPU (different
 *     streams without an ordering between them) race; order them on one stream or with events.
 *     Nothing has to be cleared between calls: every record a call reads it has written first. */
size_t sl_noalloc_scratch_bytes(void);
sl_status sl_span_attention_decode_noalloc(const sl_params* p, const void* Q, const void* K,
                                           const void* V, const int32_t* idx, void* O, float* LSE,
                                           void* hip_stream);

/* Span-attention with the paper's combination step (Section 3.4, eq. (5) and (6); Algorithm 1:
 * DedupConcat + Attention per selected span, Softmax over the selected scores, weighted sum).
 * For each (h, r) and each non-empty slot t of idx: A_t = softmax attention of the query over
 * span idx[h][r][t] followed by the local window [c*S, i] (its own softmax, logits
 * scale * <Q, K_j>); O = sum_t alpha_t A_t with alpha = softmax over the non-empty slots of
 * scores[h][r][t] (the raw search scores, as eq. (6) uses them).  A row without a non-empty slot
 * gets the attention over its local window (Algorithm 1's empty-selection branch).
 *   idx     in: as for sl_span_attention_* (entries < 0 or >= c are empty slots).
 *   scores  in: [Hq][Lq][topk] float, the `scores` output of span-search for the same idx; only
 *           the entries of non-empty slots are read and they must be finite.
 *   O       out: [Hq][Lq][D] in the input dtype.  (No LSE: the output is a mixture of softmaxes.)
 * Workspace: the same as the span-attention entry point of the same form
 * (SL_OP_ATTENTION_PREFILL / SL_OP_ATTENTION_DECODE).  The decode form requires Lq == 1. */
sl_status sl_span_attention_combined_prefill(const sl_params* p, const void* Q, const void* K,
                                             const void* V, const int32_t* idx, const float* scores,
                                             void* O, void* ws, size_t ws_bytes, void* hip_stream);
sl_status sl_span_attention_combined_decode(const sl_params* p, const void* Q, const void* K,
                                            const void* V, const int32_t* idx, const float* scores,
                                            void* O, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- The paper's own geometry, decode form (Section 3.3 with Fig. 3; Algorithm 1), p = 1/2.
 * For the query at position i = q_pos0 = L - 1 (Lq must be 1; S of sl_params is ignored):
 *   anchors      t_s = i - (s+1)^2 + 1, s = 0, 1, ..., t_s >= 0;
 *   window       W = [max(0, i - window + 1), i]  (window = 0: none); anchors inside W are not
 *                candidates.  For gap-free coverage choose window = m^2 - 1 (the paper's 1088), so
 *                that the first candidate is the token just before W;
 *   spans        S_t = [max(0, t - backward_factor * l), min(i, t + forward_factor * l)],
 *                l = ceil(sqrt(i)). */
typedef struct sl_anchor_geometry {
  int64_t window;
  int32_t backward_factor; /* b >= 0 */
  int32_t forward_factor;  /* f >= 0 */
  int32_t search_root;     /* 1/p: 0 or 2 = the geometry above (p = 1/2); 3 = the exponent split
                              (1/3, 2/3) of Section 5 in the general-p formulas of Section 3.3:
                              anchors t_s = i - (s+1)^3 + 1, l = ceil(i^(2/3)), window = m^3 - 1
                              for gap-free coverage, b >= 3 to reach every key */
  int32_t reserved;        /* 0 */
} sl_anchor_geometry;

/* Bytes of scratch sl_anchor_attention_decode needs (SL_WORKSPACE_INVALID if the arguments are invalid). */
size_t sl_anchor_workspace_bytes(const sl_params* p, const sl_anchor_geometry* g);

/* Span-search over the candidate anchors (eq. (2)-(3) with K_a = K: the key of anchor t is
 * K[kv][t]).
 *   anchors out: [Hq][topk] int32, the token positions of the min(topk, #candidates) best
 *           anchors per head, nearest anchor (lowest stride index) first, remaining slots -1.
 *           Ties in score go to the nearer anchor.
 *   scores  out, optional: fp32 score of the anchor in the same slot, -inf in empty slots.
 * At most 4096 candidate anchors (i < 2^24). */
sl_status sl_anchor_search_decode(const sl_params* p, const sl_anchor_geometry* g, const void* Qs,
                                  const void* K, int32_t* anchors, float* scores, void* hip_stream);

/* Span-attention and combination over the selected anchors (Algorithm 1): per non-empty slot,
 * A_t = softmax attention over DedupConcat(S_t, W) (every token once, logits scale * <Q, K_j>),
 * O = sum_t alpha_t A_t with alpha = softmax of scores over the non-empty slots; no non-empty
 * slot: attention over W (zeros if there is no window either).
 *   anchors in: as produced by sl_anchor_search_decode (entries < 0 or > i are empty slots).
 *   scores  in: [Hq][topk] float, finite in non-empty slots.   O out: [Hq][1][D]. */
sl_status sl_anchor_attention_decode(const sl_params* p, const sl_anchor_geometry* g, const void* Q,
                                     const void* K, const void* V, const int32_t* anchors,
                                     const float* scores, void* O, void* ws, size_t ws_bytes,
                                     void* hip_stream);

/* ---- The same geometry, prefill form: every query row r (position i = q_pos0 + r) has its own
 * anchors, its own l = ceil(sqrt(i)) and its own window, exactly as in the decode form above
 * (Section 3.3, Algorithm 1).  S of sl_params is ignored.
 *   anchors: [Hq][Lq][topk] int32, scores: [Hq][Lq][topk] float, O: [Hq][Lq][D]; slot meaning and
 *   tie rule as in the decode form.  At most 12288 candidate anchors per row.
 * Span-search is row-stationary (one wavefront per query row), fp32 or bf16, no workspace.
 * Span-attention + combination has two forms:
 *   - with a workspace of sl_anchor_prefill_workspace_bytes (bf16, D = 128, window >= 1, topk >= 1):
 *     the matrix-core form, which follows Section 4.3's prefilling kernel: (row, slot) pairs are
 *     bucketed by the key block that holds the last token of their span (blocks of 64 .. 4096
 *     tokens, chosen from the problem size), the rows of a bucket share one sliding K/V range with
 *     per-row masks, the window is a banded flash kernel, and a gated merge combines the partials;
 *   - with ws == NULL, or where sl_anchor_prefill_workspace_bytes returns 0: row-stationary kernels
 *     (fp32 or bf16, any shape), no workspace. */
sl_status sl_anchor_search_prefill(const sl_params* p, const sl_anchor_geometry* g, const void* Qs,
                                   const void* K, int32_t* anchors, float* scores, void* hip_stream);
/* Scratch bytes of the matrix-core form (0: that form does not apply to these parameters;
 * SL_WORKSPACE_INVALID: invalid parameters). */
size_t sl_anchor_prefill_workspace_bytes(const sl_params* p, const sl_anchor_geometry* g);
sl_status sl_anchor_attention_prefill(const sl_params* p, const sl_anchor_geometry* g, const void* Q,
                                      const void* K, const void* V, const int32_t* anchors,
                                      const float* scores, void* O, void* ws, size_t ws_bytes,
                                      void* hip_stream);

/* ---- Batched decode: one step for B independent sequences in three launches (Section 4.3's
 * decoding path serves a batch of sequences; the grid gains a sequence dimension).  Every
 * sequence b has its own cache of seq[b].L tokens (its query sits at position L - 1) and its own
 * tensors; heads, D, S, topk, dtype, scale and the element strides are common and come from p
 * (p->L must be the largest L of the batch, p->Lq = 1, p->q_pos0 = p->L - 1; a head stride given
 * as 0 means "packed for this sequence's own L").  `seqs` is an array of B records in DEVICE
 * memory, read by the kernels: its contents cannot be validated by the host, so every pointer in
 * it must be valid and 16-byte aligned and 1 <= L <= p->L must hold -- that is the caller's
 * responsibility.  Profile events are not recorded by the batched entry points. */
typedef struct sl_decode_seq {
  const void* Qs;  /* search query   [Hq][1][D]                                   */
  const void* Q;   /* attention query [Hq][1][D]                                  */
  const void* K;   /* [Hkv][L][D]                                                 */
  const void* V;   /* [Hkv][L][D]                                                 */
  const void* Ks;  /* packed span keys [Hkv][ceil(L/S)][D], or NULL (keys from K) */
  int32_t* idx;    /* out (search) / in (attention): [Hq][1][topk]                */
  float* scores;   /* out, optional: [Hq][1][topk]                                */
  void* O;         /* out: [Hq][1][D]                                             */
  float* LSE;      /* out: [Hq][1]                                                */
  int64_t L;       /* tokens in this sequence's cache, current token included     */
} sl_decode_seq;

/* Scratch bytes of sl_span_attention_decode_batched for B sequences (SL_WORKSPACE_INVALID if invalid). */
size_t sl_decode_batched_workspace_bytes(const sl_params* p, int32_t B);

/* sl_span_search_decode for every sequence of the batch: fills seq[b].idx (and scores).
 * Limits as for one sequence (at most 12288 spans in the longest cache). */
sl_status sl_span_search_decode_batched(const sl_params* p, const sl_decode_seq* seqs, int32_t B,
                                        void* hip_stream);

/* sl_span_attention_decode for every sequence of the batch on seq[b].idx: fills seq[b].O, LSE. */
sl_status sl_span_attention_decode_batched(const sl_params* p, const sl_decode_seq* seqs, int32_t B,
                                           void* ws, size_t ws_bytes, void* hip_stream);

/* The combination form (sl_span_attention_combined_decode) for every sequence of the batch: the
 * gate is seq[b].scores as written by sl_span_search_decode_batched (required), O is written, LSE
 * is not.  Workspace: sl_decode_batched_workspace_bytes. */
sl_status sl_span_attention_combined_decode_batched(const sl_params* p, const sl_decode_seq* seqs,
                                                    int32_t B, void* ws, size_t ws_bytes,
                                                    void* hip_stream);

/* The paper's own geometry (sl_anchor_search_decode / sl_anchor_attention_decode) for a batch:
 * window, span factors and exponent are common (g), every sequence's query sits at its own
 * L - 1, so its anchors, its span base length l(L - 1) and its window follow from its own
 * length.  p->S is ignored, seq[b].Ks is not read; seq[b].idx receives / supplies anchor TOKEN
 * positions, seq[b].scores the gate (required); O is written, LSE is not. */
size_t sl_anchor_batched_workspace_bytes(const sl_params* p, const sl_anchor_geometry* g, int32_t B);
sl_status sl_anchor_search_decode_batched(const sl_params* p, const sl_anchor_geometry* g,
                                          const sl_decode_seq* seqs, int32_t B, void* hip_stream);
sl_status sl_anchor_attention_decode_batched(const sl_params* p, const sl_anchor_geometry* g,
                                             const sl_decode_seq* seqs, int32_t B, void* ws,
                                             size_t ws_bytes, void* hip_stream);

/* Static, human-readable name of a status code. */
const char* sl_status_string(sl_status status);

/* Library version as major * 10000 + minor * 100 + patch. */
int sl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SL_H_ */
