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
typedef int (*prefill_fn)(const qs_cache *, const void *, const void *, int64_t, int32_t, void *);
typedef int (*append_fn)(const qs_cache *, const void *, const void *, int32_t, void *);
typedef int (*verify_fn)(const qs_cache *, const void *, int32_t, void *, float, void *, size_t, float *, void *);
typedef int (*static_fn)(const qs_cache *, const void *, int32_t, int32_t, void *, float, float *, void *);
typedef int (*export_fn)(const qs_cache *, int32_t, int32_t, int32_t, void *, void *, void *, void *, void *, void *,
                         void *, void *, void *);

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
  prefill_fn prefill;
  append_fn append;
  verify_fn verify;
  static_fn attn_static;
  export_fn export_codes;
  /* POSIX's way to turn dlsym's object pointer into a function pointer */
  *(void **)(&version) = dlsym(lib, "qs_version");
  *(void **)(&err) = dlsym(lib, "qs_strerror");
  *(void **)(&ws) = dlsym(lib, "qs_workspace_bytes");
  *(void **)(&draft) = dlsym(lib, "qs_attn_draft");
  *(void **)(&flush) = dlsym(lib, "qs_quantize_flush");
  *(void **)(&prefill) = dlsym(lib, "qs_quantize_prefill");
  *(void **)(&append) = dlsym(lib, "qs_append");
  *(void **)(&verify) = dlsym(lib, "qs_attn_verify");
  *(void **)(&attn_static) = dlsym(lib, "qs_attn_static");
  *(void **)(&export_codes) = dlsym(lib, "qs_export_codes");
  CHECK(version && err && ws && draft && flush && prefill && append && verify && attn_static && export_codes);
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
  /* every entry point's argument checks, none of which reaches the GPU */
  CHECK(flush(&c, 256, NULL) == QS_ERR_RANGE);                                       /* n_buf[1] = 130 < 256 */
  CHECK(prefill(&c, NULL, (void *)0x80000, 2048, 128, NULL) == QS_ERR_NULL);
  CHECK(prefill(&c, (void *)0x80008, (void *)0x90000, 2048, 128, NULL) == QS_ERR_ALIGN);
  CHECK(prefill(&c, (void *)0x80000, (void *)0x90000, 64, 128, NULL) == QS_ERR_RANGE);   /* stride < n_tokens */
  CHECK(prefill(&c, (void *)0x80000, (void *)0x90000, 2048, 0, NULL) == QS_OK);
  CHECK(append(&c, (void *)0x80000, NULL, 1, NULL) == QS_ERR_NULL);
  CHECK(append(&c, (void *)0x80000, (void *)0x90000, 9, NULL) == QS_ERR_RANGE);          /* 256 + 9 > buf_cap */
  CHECK(append(&c, (void *)0x80000, (void *)0x90000, 0, NULL) == QS_OK);
  CHECK(verify(&c, (void *)0x50000, QS_MAX_NQ + 1, (void *)0x60000, 0.1f, (void *)0x70000, bytes, NULL, NULL) == QS_ERR_UNSUPPORTED);
  CHECK(verify(&c, (void *)0x50000, 5, (void *)0x60000, -1.0f, (void *)0x70000, bytes, NULL, NULL) == QS_ERR_RANGE);
  CHECK(verify(&c, (void *)0x50000, 5, (void *)0x60004, 0.1f, (void *)0x70000, bytes, NULL, NULL) == QS_ERR_ALIGN);
  CHECK(attn_static(&c, (void *)0x50000, 1, 2, (void *)0x60000, 0.1f, NULL, NULL) == QS_ERR_RANGE);
  CHECK(attn_static(&c, (void *)0x50000, 3, 0, (void *)0x60000, 0.1f, NULL, NULL) == QS_ERR_UNSUPPORTED);
  CHECK(attn_static(&c, NULL, 1, 0, (void *)0x60000, 0.1f, NULL, NULL) == QS_ERR_NULL);
  CHECK(export_codes(&c, 2, 0, 128, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == QS_ERR_RANGE);
  CHECK(export_codes(&c, 0, 0, 100, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == QS_ERR_RANGE);
  n_buf[0] = 2;
  CHECK(verify(&c, (void *)0x50000, 5, (void *)0x60000, 0.1f, (void *)0x70000, bytes, NULL, NULL) == QS_ERR_RANGE);   /* n_buf < nq */
  n_buf[0] = 256;
  c.compute_units = -3;
  CHECK(ws(&c, 1) == 0 && flush(&c, 128, NULL) == QS_ERR_RANGE);
  c.compute_units = 0, c.flags = 0x40;
  CHECK(flush(&c, 128, NULL) == QS_ERR_RANGE);
  c.flags = QS_FLAG_FIXED_RANGES;
  CHECK(ws(&c, 5) == bytes);
  c.n_q_heads = 7;
  CHECK(flush(&c, 128, NULL) == QS_ERR_SHAPE);
  puts("ok");
  return 0;
}
