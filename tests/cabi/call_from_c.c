/* Loads the library from plain C through its header and exercises the host-only entry points:
 * version, status strings, workspace sizing and argument validation (nothing is launched). */
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>

#include "sl.h"

typedef int (*version_fn)(void);
typedef const char* (*status_fn)(int);
typedef size_t (*ws_fn)(const sl_params*, int);
typedef sl_status (*search_fn)(const sl_params*, const void*, const void*, const void*, int32_t*, float*,
                               void*, size_t, void*);

int main(int argc, char** argv) {
  if (argc < 2) return 2;
  void* lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
  if (!lib) {
    fprintf(stderr, "dlopen: %s\n", dlerror());
    return 3;
  }
  version_fn version = (version_fn)dlsym(lib, "sl_version");
  status_fn status = (status_fn)dlsym(lib, "sl_status_string");
  ws_fn ws_bytes = (ws_fn)dlsym(lib, "sl_workspace_bytes");
  search_fn search = (search_fn)dlsym(lib, "sl_span_search_decode");
  if (!version || !status || !ws_bytes || !search) return 4;

  sl_params p;
  memset(&p, 0, sizeof p);
  p.L = 1 << 20;
  p.Lq = 1;
  p.q_pos0 = p.L - 1;
  p.Hq = 32;
  p.Hkv = 4;
  p.D = 128;
  p.S = 1024;
  p.topk = 16;
  p.dtype = SL_BF16;
  const size_t need = ws_bytes(&p, SL_OP_ATTENTION_DECODE);
  /* a null query pointer must be rejected on the host, before anything is enqueued */
  const sl_status st = search(&p, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL);
  printf("version=%d ok=%s bad=%s ws=%zu st=%d\n", version(), status(SL_OK), status(st), need, (int)st);
  return (version() >= 100 && need > 0 && st == SL_ERR_INVALID_ARG && strcmp(status(SL_OK), "SL_OK") == 0) ? 0 : 1;
}
