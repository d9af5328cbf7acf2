/* Drives the host-side validation layer of the library (no GPU needed: every call below must be
 * rejected before anything is enqueued).  Built with AddressSanitizer + UBSan against the
 * sanitizer build of the library, so that an out-of-bounds access or undefined operation on any
 * rejection path aborts the program.  Prints the number of checks that passed; exit code 0 = all. */
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>

#include "sl.h"

typedef size_t (*ws_fn)(const sl_params*, int);
typedef sl_status (*search_fn)(const sl_params*, const void*, const void*, const void*, int32_t*, float*,
                               void*, size_t, void*);
typedef sl_status (*attn_fn)(const sl_params*, const void*, const void*, const void*, const int32_t*, void*,
                             float*, void*, size_t, void*);
typedef sl_status (*noalloc_fn)(const sl_params*, const void*, const void*, const void*, const int32_t*,
                                void*, float*, void*);
typedef sl_status (*batched_fn)(const sl_params*, const sl_decode_seq*, int32_t, void*, size_t, void*);
typedef size_t (*anchor_ws_fn)(const sl_params*, const sl_anchor_geometry*);
typedef const char* (*status_fn)(sl_status);

static int failures = 0, checks = 0;
#define EXPECT(cond)                                                    \
  do {                                                                  \
    ++checks;                                                           \
    if (!(cond)) {                                                      \
      ++failures;                                                       \
      fprintf(stderr, "line %d: %s\n", __LINE__, #cond);                \
    }                                                                   \
  } while (0)

static sl_params good(void) {
  sl_params p;
  memset(&p, 0, sizeof p);
  p.L = 4096;
  p.Lq = 4096;
  p.Hq = 8;
  p.Hkv = 2;
  p.D = 128;
  p.S = 64;
  p.topk = 4;
  p.dtype = SL_BF16;
  return p;
}

int main(int argc, char** argv) {
  if (argc < 2) return 2;
  void* lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
  if (!lib) {
    fprintf(stderr, "dlopen: %s\n", dlerror());
    return 3;
  }
  ws_fn ws_bytes = (ws_fn)dlsym(lib, "sl_workspace_bytes");
  search_fn search_p = (search_fn)dlsym(lib, "sl_span_search_prefill");
  search_fn search_d = (search_fn)dlsym(lib, "sl_span_search_decode");
  attn_fn attn_p = (attn_fn)dlsym(lib, "sl_span_attention_prefill");
  attn_fn attn_d = (attn_fn)dlsym(lib, "sl_span_attention_decode");
  noalloc_fn attn_n = (noalloc_fn)dlsym(lib, "sl_span_attention_decode_noalloc");
  batched_fn attn_b = (batched_fn)dlsym(lib, "sl_span_attention_decode_batched");
  anchor_ws_fn anchor_ws = (anchor_ws_fn)dlsym(lib, "sl_anchor_workspace_bytes");
  status_fn status = (status_fn)dlsym(lib, "sl_status_string");
  if (!ws_bytes || !search_p || !search_d || !attn_p || !attn_d || !attn_n || !attn_b || !anchor_ws || !status)
    return 4;
  void* const fake = (void*)0x1000;   /* non-null, aligned, never dereferenced on a rejection path */
  void* const fake_ws = (void*)0x10000;

  sl_params p = good();
  EXPECT(ws_bytes(NULL, SL_OP_ATTENTION_PREFILL) == SL_WORKSPACE_INVALID);
  EXPECT(ws_bytes(&p, 17) == SL_WORKSPACE_INVALID);
  EXPECT(ws_bytes(&p, SL_OP_SEARCH_PREFILL) == 0);
  EXPECT(ws_bytes(&p, SL_OP_ATTENTION_PREFILL) > 0 && ws_bytes(&p, SL_OP_ATTENTION_PREFILL) != SL_WORKSPACE_INVALID);

  /* sizes at the edge of the integer ranges: the size arithmetic must not overflow */
  p = good();
  p.L = p.Lq = (int64_t)1 << 40;
  (void)ws_bytes(&p, SL_OP_ATTENTION_PREFILL);
  EXPECT(attn_p(&p, fake, fake, fake, fake, fake, fake, fake_ws, 0, NULL) != SL_OK);
  p = good();
  p.Hq = 2147483640;
  p.Hkv = 1;
  EXPECT(attn_p(&p, fake, fake, fake, fake, fake, fake, fake_ws, (size_t)1 << 40, NULL) == SL_ERR_UNSUPPORTED);
  p = good();
  p.S = 2147483647;
  p.L = p.Lq = 10;
  (void)ws_bytes(&p, SL_OP_ATTENTION_DECODE);
  p = good();
  p.q_stride_t = ((int64_t)1 << 62);
  (void)ws_bytes(&p, SL_OP_ATTENTION_PREFILL);

  /* every field out of range */
  const struct { int field; int64_t value; sl_status want; } bad[] = {
      {0, 0, SL_ERR_INVALID_ARG},  {1, 0, SL_ERR_INVALID_ARG},   {2, -1, SL_ERR_INVALID_ARG},
      {3, 0, SL_ERR_INVALID_ARG},  {4, 3, SL_ERR_INVALID_ARG},   {5, 96, SL_ERR_UNSUPPORTED},
      {6, 0, SL_ERR_INVALID_ARG},  {7, -1, SL_ERR_INVALID_ARG},  {7, SL_MAX_TOPK + 1, SL_ERR_UNSUPPORTED},
      {8, 9, SL_ERR_INVALID_ARG},
  };
  for (size_t i = 0; i < sizeof bad / sizeof bad[0]; ++i) {
    p = good();
    switch (bad[i].field) {
      case 0: p.L = bad[i].value; break;
      case 1: p.Lq = bad[i].value; break;
      case 2: p.q_pos0 = bad[i].value; break;
      case 3: p.Hq = (int32_t)bad[i].value; break;
      case 4: p.Hkv = (int32_t)bad[i].value; break;
      case 5: p.D = (int32_t)bad[i].value; break;
      case 6: p.S = (int32_t)bad[i].value; break;
      case 7: p.topk = (int32_t)bad[i].value; break;
      default: p.dtype = (int32_t)bad[i].value; break;
    }
    EXPECT(search_p(&p, fake, fake, fake, fake, NULL, fake_ws, (size_t)1 << 40, NULL) == bad[i].want);
    EXPECT(attn_p(&p, fake, fake, fake, fake, fake, fake, fake_ws, (size_t)1 << 40, NULL) == bad[i].want);
    EXPECT(ws_bytes(&p, SL_OP_ATTENTION_PREFILL) == SL_WORKSPACE_INVALID);
  }

  /* pointers: null, misaligned; workspace: missing, short, misaligned */
  p = good();
  EXPECT(search_p(&p, NULL, fake, fake, fake, NULL, NULL, 0, NULL) == SL_ERR_INVALID_ARG);
  EXPECT(search_p(&p, fake, NULL, NULL, fake, NULL, NULL, 0, NULL) == SL_ERR_INVALID_ARG);
  EXPECT(search_p(&p, (void*)0x1004, fake, fake, fake, NULL, NULL, 0, NULL) == SL_ERR_INVALID_ARG);
  const size_t need = ws_bytes(&p, SL_OP_ATTENTION_PREFILL);
  EXPECT(attn_p(&p, fake, fake, fake, fake, fake, fake, NULL, 0, NULL) == SL_ERR_WORKSPACE);
  EXPECT(attn_p(&p, fake, fake, fake, fake, fake, fake, fake_ws, need - 1, NULL) == SL_ERR_WORKSPACE);
  EXPECT(attn_p(&p, fake, fake, fake, fake, fake, fake, (void*)0x10010, need, NULL) == SL_ERR_WORKSPACE);
  EXPECT(attn_p(&p, fake, fake, fake, fake, fake, NULL, fake_ws, need, NULL) == SL_ERR_INVALID_ARG);

  /* decode forms need Lq == 1; the array of the no-alloc entry point has a size limit */
  EXPECT(search_d(&p, fake, fake, fake, fake, NULL, NULL, 0, NULL) == SL_ERR_INVALID_ARG);
  EXPECT(attn_d(&p, fake, fake, fake, fake, fake, fake, fake_ws, (size_t)1 << 40, NULL) == SL_ERR_INVALID_ARG);
  EXPECT(attn_n(&p, fake, fake, fake, fake, fake, fake, NULL) == SL_ERR_INVALID_ARG);
  p = good();
  p.L = 2 * 16384;
  p.Lq = 1;
  p.q_pos0 = p.L - 1;
  p.Hq = 32;
  p.Hkv = 4;
  p.S = 16384;
  p.topk = 32;
  EXPECT(attn_n(&p, fake, fake, fake, fake, fake, fake, NULL) == SL_ERR_UNSUPPORTED);
  EXPECT(attn_n(&p, fake, fake, fake, NULL, fake, fake, NULL) == SL_ERR_INVALID_ARG);
  EXPECT(attn_b(&p, NULL, 2, fake_ws, (size_t)1 << 40, NULL) == SL_ERR_INVALID_ARG);
  EXPECT(attn_b(&p, (const sl_decode_seq*)fake, 0, fake_ws, (size_t)1 << 40, NULL) == SL_ERR_INVALID_ARG);

  /* the paper's geometry */
  sl_anchor_geometry g = {1088, 4, 2, 2, 0};
  EXPECT(anchor_ws(&p, &g) != SL_WORKSPACE_INVALID);
  g.search_root = 5;
  EXPECT(anchor_ws(&p, &g) == SL_WORKSPACE_INVALID);
  EXPECT(anchor_ws(&p, NULL) == SL_WORKSPACE_INVALID);

  for (int s = 0; s < 8; ++s) EXPECT(status((sl_status)s) != NULL && strlen(status((sl_status)s)) > 0);
  printf("checks=%d failures=%d\n", checks, failures);
  return failures ? 1 : 0;
}
