/* The public header compiles as plain C99 and the library can be driven from C without Python:
   version, error strings, workspace sizing and argument validation (none of which touch the GPU).
   Built and run by tests/test_abi.py; prints "ok" and exits 0 on success. */
#include <dlfcn.h>
#include <stdio.h>
#include <string.h>

#include "quantspec.h"

#define CHECK(cond)                                             \
  do {                                                          \
    if (!(cond)) {                                              \
      fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                 \
    }                                                           \
  } while (0)

typedef int (*version_fn)(void);
typedef const char *(*strerror_fn)(int);
typedef size_t (*ws_fn)(const qs_cache *, int32_t);
typedef int (*draft_fn)(const qs_cache *, const void *, void *, float, void *, size_t, float *, void *);
typedef int (*flush_fn)(const qs_cache *, int32_t, void *);

int main(int argc, char **argv) {
  CHECK(argc == 2);
  void *lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
  if (lib == NULL) {
    fprintf(stderr, "dlopen: %s\n", dlerror());
    return 1;
  }
  version_fn version;
  strerror_fn err;
  ws_fn ws;
  draft_fn draft;
  flush_fn flush;
  /* POSIX's way to turn dlsym's object pointer into a function pointer */
  *(void **)(&version) = dlsym(lib, "qs_version");
  *(void **)(&err) = dlsym(lib, "qs_strerror");
  *(void **)(&ws) = dlsym(lib, "qs_workspace_bytes");
  *(void **)(&draft) = dlsym(lib, "qs_attn_draft");
  *(void **)(&flush) = dlsym(lib, "qs_quantize_flush");
  CHECK(version && err && ws && draft && flush);
  CHECK(version() >= 100);
  CHECK(strcmp(err(QS_OK), "ok") == 0);

  int32_t n_quant[2] = {512, 1024}, n_buf[2] = {256, 130};
  qs_cache c;
  memset(&c, 0, sizeof c);
  c.batch = 2, c.n_q_heads = 8, c.n_kv_heads = 2, c.head_dim = 128, c.group = 128;
  c.q_cap = 1024, c.buf_cap = 264;
  c.upper = (void *)0x10000, c.lower = (void *)0x20000;   /* never dereferenced: validation only */
  c.k_buf = (void *)0x30000, c.v_buf = (void *)0x40000;
  c.n_quant = n_quant, c.n_buf = n_buf;

  const size_t bytes = ws(&c, 5);
  CHECK(bytes > 0 && bytes % (130 * sizeof(float)) == 0);
  CHECK(ws(&c, QS_MAX_NQ + 1) == 0);
  CHECK(draft(&c, (void *)0x50000, (void *)0x60000, 0.1f, NULL, 0, NULL, NULL) == QS_ERR_WORKSPACE);
  CHECK(draft(&c, NULL, (void *)0x60000, 0.1f, (void *)0x70000, bytes, NULL, NULL) == QS_ERR_NULL);
  c.head_dim = 64;
  CHECK(draft(&c, (void *)0x50000, (void *)0x60000, 0.1f, (void *)0x70000, bytes, NULL, NULL) == QS_ERR_UNSUPPORTED);
  c.head_dim = 128;
  CHECK(flush(&c, 100, NULL) == QS_ERR_RANGE);
  CHECK(flush(&c, 0, NULL) == QS_OK);
  puts("ok");
  return 0;
}
