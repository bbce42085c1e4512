/* Drives the library on a GPU from plain C99, without Python: prefill quantization, draft and verify
   attention, a flush, and the export of one unit's codes, checked against a fixture that
   tests/c_abi/make_fixture.py wrote from the CPU oracle.  The HIP runtime is reached through dlopen
   (allocation, copies, synchronization only).  Built and run by tests/test_gpu_c_abi.py.
   usage: gpu_run <libquantspec.so> <fixture>; prints "ok" and exits 0 on success. */
#include <dlfcn.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "quantspec.h"

#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                  \
    }                                                            \
  } while (0)

typedef int (*hip_malloc_fn)(void **, size_t);
typedef int (*hip_free_fn)(void *);
typedef int (*hip_memcpy_fn)(void *, const void *, size_t, int);
typedef int (*hip_memset_fn)(void *, int, size_t);
typedef int (*hip_sync_fn)(void);
enum { H2D = 1, D2H = 2 };

typedef size_t (*ws_fn)(const qs_cache *, int32_t);
typedef int (*prefill_fn)(const qs_cache *, const void *, const void *, int64_t, int32_t, void *);
typedef int (*flush_fn)(const qs_cache *, int32_t, void *);
typedef int (*draft_fn)(const qs_cache *, const void *, void *, float, void *, size_t, float *, void *);
typedef int (*verify_fn)(const qs_cache *, const void *, int32_t, void *, float, void *, size_t, float *, void *);
typedef int (*static_fn)(const qs_cache *, const void *, int32_t, int32_t, void *, float, float *, void *);
typedef int (*export_fn)(const qs_cache *, int32_t, int32_t, int32_t, void *, void *, void *, void *, void *, void *,
                         void *, void *, void *);

static float half_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h >> 15) << 31, exp = (h >> 10) & 31, man = h & 1023;
  float f;
  uint32_t bits;
  if (exp == 0) return (sign ? -1.0f : 1.0f) * (float)man * 5.9604644775390625e-8f;   /* subnormal: man * 2^-24 */
  bits = sign | ((exp == 31 ? 255u : exp + 112u) << 23) | (man << 13);
  memcpy(&f, &bits, sizeof f);
  return f;
}

/* max over output vectors of max_d |gpu - ref| / max_d |ref| */
static double rel_err(const uint16_t *gpu, const double *ref, size_t vectors) {
  double worst = 0.0;
  for (size_t i = 0; i < vectors; ++i) {
    double num = 0.0, den = 0.0;
    for (int d = 0; d < 128; ++d) {
      const double r = ref[i * 128 + d], e = fabs((double)half_to_float(gpu[i * 128 + d]) - r);
      if (e > num) num = e;
      if (fabs(r) > den) den = fabs(r);
    }
    if (num / den > worst) worst = num / den;
  }
  return worst;
}

int main(int argc, char **argv) {
  CHECK(argc == 3);
  void *hip = dlopen("libamdhip64.so", RTLD_NOW | RTLD_GLOBAL);
  if (hip == NULL) {
    fprintf(stderr, "dlopen libamdhip64.so: %s\n", dlerror());
    return 1;
  }
  void *lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
  if (lib == NULL) {
    fprintf(stderr, "dlopen %s: %s\n", argv[1], dlerror());
    return 1;
  }
  hip_malloc_fn hip_malloc;
  hip_free_fn hip_free;
  hip_memcpy_fn hip_memcpy;
  hip_memset_fn hip_memset;
  hip_sync_fn hip_sync;
  ws_fn ws_bytes;
  prefill_fn prefill;
  flush_fn flush;
  draft_fn draft;
  verify_fn verify;
  static_fn attn_static;
  export_fn export_codes;
  *(void **)(&hip_malloc) = dlsym(hip, "hipMalloc");
  *(void **)(&hip_free) = dlsym(hip, "hipFree");
  *(void **)(&hip_memcpy) = dlsym(hip, "hipMemcpy");
  *(void **)(&hip_memset) = dlsym(hip, "hipMemset");
  *(void **)(&hip_sync) = dlsym(hip, "hipDeviceSynchronize");
  *(void **)(&ws_bytes) = dlsym(lib, "qs_workspace_bytes");
  *(void **)(&prefill) = dlsym(lib, "qs_quantize_prefill");
  *(void **)(&flush) = dlsym(lib, "qs_quantize_flush");
  *(void **)(&draft) = dlsym(lib, "qs_attn_draft");
  *(void **)(&verify) = dlsym(lib, "qs_attn_verify");
  *(void **)(&attn_static) = dlsym(lib, "qs_attn_static");
  *(void **)(&export_codes) = dlsym(lib, "qs_export_codes");
  CHECK(hip_malloc && hip_free && hip_memcpy && hip_memset && hip_sync);
  CHECK(ws_bytes && prefill && flush && draft && verify && attn_static && export_codes);

  /* ---- fixture ---- */
  FILE *f = fopen(argv[2], "rb");
  CHECK(f != NULL);
  int32_t hdr[8];
  CHECK(fread(hdr, sizeof hdr, 1, f) == 1 && hdr[0] == 0x51534658);
  const int B = hdr[1], Hq = hdr[2], Hkv = hdr[3], Tq = hdr[4], nb = hdr[5], nq = hdr[6], n_flush = hdr[7];
  const int T = Tq + nb, T2 = Tq + n_flush;
  const size_t kv_elems = (size_t)B * Hkv * T * 128, qd_elems = (size_t)B * Hq * 128, qv_elems = qd_elems * nq;
  uint16_t *k = malloc(kv_elems * 2), *v = malloc(kv_elems * 2), *qd = malloc(qd_elems * 2), *qv = malloc(qv_elems * 2);
  double *ref_d = malloc(qd_elems * 8), *ref_v = malloc(qv_elems * 8), *ref_v2 = malloc(qv_elems * 8);
  uint8_t *ku = malloc((size_t)T2 * 128), *vu = malloc((size_t)T2 * 128);
  int8_t *kl = malloc((size_t)T2 * 128), *vl = malloc((size_t)T2 * 128);
  uint16_t *ks = malloc((size_t)T2 * 2), *kz = malloc((size_t)T2 * 2), *vs = malloc((size_t)T2 * 2), *vz = malloc((size_t)T2 * 2);
  CHECK(k && v && qd && qv && ref_d && ref_v && ref_v2 && ku && vu && kl && vl && ks && kz && vs && vz);
  CHECK(fread(k, 2, kv_elems, f) == kv_elems && fread(v, 2, kv_elems, f) == kv_elems);
  CHECK(fread(qd, 2, qd_elems, f) == qd_elems && fread(qv, 2, qv_elems, f) == qv_elems);
  CHECK(fread(ref_d, 8, qd_elems, f) == qd_elems && fread(ref_v, 8, qv_elems, f) == qv_elems);
  CHECK(fread(ku, 1, (size_t)T2 * 128, f) == (size_t)T2 * 128 && fread(kl, 1, (size_t)T2 * 128, f) == (size_t)T2 * 128);
  CHECK(fread(vu, 1, (size_t)T2 * 128, f) == (size_t)T2 * 128 && fread(vl, 1, (size_t)T2 * 128, f) == (size_t)T2 * 128);
  CHECK(fread(ks, 2, (size_t)T2, f) == (size_t)T2 && fread(kz, 2, (size_t)T2, f) == (size_t)T2);   /* T2/128 groups x 128 */
  CHECK(fread(vs, 2, (size_t)T2, f) == (size_t)T2 && fread(vz, 2, (size_t)T2, f) == (size_t)T2);
  CHECK(fread(ref_v2, 8, qv_elems, f) == qv_elems);
  fclose(f);

  /* ---- device cache ---- */
  const int q_cap = T2, buf_cap = nb + 8;
  int32_t n_quant[QS_MAX_BATCH], n_buf[QS_MAX_BATCH];
  qs_cache c;
  memset(&c, 0, sizeof c);
  c.batch = B, c.n_q_heads = Hq, c.n_kv_heads = Hkv, c.head_dim = 128, c.group = 128;
  c.q_cap = q_cap, c.buf_cap = buf_cap;
  c.n_quant = n_quant, c.n_buf = n_buf;
  c.flags = QS_FLAG_FIXED_RANGES;
  const size_t upper_bytes = (size_t)B * Hkv * (q_cap / 32) * 4352, lower_bytes = (size_t)B * Hkv * (q_cap / 32) * 4096;
  const size_t buf_bytes = (size_t)B * Hkv * buf_cap * 128 * 2;
  void *k_src, *v_src, *q_dev, *out_dev, *ws;
  CHECK(hip_malloc(&c.upper, upper_bytes) == 0 && hip_malloc(&c.lower, lower_bytes) == 0);
  CHECK(hip_malloc(&c.k_buf, buf_bytes) == 0 && hip_malloc(&c.v_buf, buf_bytes) == 0);
  CHECK(hip_malloc(&k_src, kv_elems * 2) == 0 && hip_malloc(&v_src, kv_elems * 2) == 0);
  CHECK(hip_malloc(&q_dev, qv_elems * 2) == 0 && hip_malloc(&out_dev, qv_elems * 2) == 0);
  CHECK(hip_memset(c.upper, 0, upper_bytes) == 0 && hip_memset(c.lower, 0, lower_bytes) == 0);
  CHECK(hip_memset(c.k_buf, 0, buf_bytes) == 0 && hip_memset(c.v_buf, 0, buf_bytes) == 0);
  CHECK(hip_memcpy(k_src, k, kv_elems * 2, H2D) == 0 && hip_memcpy(v_src, v, kv_elems * 2, H2D) == 0);
  for (int b = 0; b < B; ++b) n_quant[b] = 0, n_buf[b] = 0;
  const size_t ws_size = ws_bytes(&c, nq);
  CHECK(ws_size > 0 && ws_bytes(&c, 1) <= ws_size);
  CHECK(hip_malloc(&ws, ws_size) == 0);

  /* prefill: the first Tq tokens go to the planes, the rest to the buffer */
  CHECK(prefill(&c, k_src, v_src, T, Tq, NULL) == QS_OK);
  for (int b = 0; b < B; ++b) {
    n_quant[b] = Tq, n_buf[b] = nb;
    for (int h = 0; h < Hkv; ++h) {
      const size_t src = (((size_t)b * Hkv + h) * T + Tq) * 128, dst = ((size_t)b * Hkv + h) * buf_cap * 128;
      CHECK(hip_memcpy((uint16_t *)c.k_buf + dst, k + src, (size_t)nb * 256, H2D) == 0);
      CHECK(hip_memcpy((uint16_t *)c.v_buf + dst, v + src, (size_t)nb * 256, H2D) == 0);
    }
  }

  /* ---- draft and verify attention ---- */
  uint16_t *out = malloc(qv_elems * 2);
  CHECK(out != NULL);
  const float sm = 1.0f / sqrtf(128.0f);
  CHECK(hip_memcpy(q_dev, qd, qd_elems * 2, H2D) == 0);
  CHECK(draft(&c, q_dev, out_dev, sm, ws, ws_size, NULL, NULL) == QS_OK);
  CHECK(hip_sync() == 0 && hip_memcpy(out, out_dev, qd_elems * 2, D2H) == 0);
  const double e_d = rel_err(out, ref_d, qd_elems / 128);
  CHECK(hip_memcpy(q_dev, qv, qv_elems * 2, H2D) == 0);
  CHECK(verify(&c, q_dev, nq, out_dev, sm, ws, ws_size, NULL, NULL) == QS_OK);
  CHECK(hip_sync() == 0 && hip_memcpy(out, out_dev, qv_elems * 2, D2H) == 0);
  const double e_v = rel_err(out, ref_v, qv_elems / 128);

  /* ---- flush, then the target pass again through the entry point with the built-in scratch ---- */
  CHECK(flush(&c, n_flush, NULL) == QS_OK);
  for (int b = 0; b < B; ++b) n_quant[b] += n_flush, n_buf[b] -= n_flush;
  CHECK(attn_static(&c, q_dev, nq, 1, out_dev, sm, NULL, NULL) == QS_OK);
  CHECK(hip_sync() == 0 && hip_memcpy(out, out_dev, qv_elems * 2, D2H) == 0);
  const double e_v2 = rel_err(out, ref_v2, qv_elems / 128);
  printf("draft %.2e  verify %.2e  verify after flush %.2e\n", e_d, e_v, e_v2);
  CHECK(e_d <= 2e-3 && e_v <= 2e-3 && e_v2 <= 2e-3);

  /* ---- codes and metadata of the last unit, prefill groups and the flushed group, bit for bit ---- */
  void *d_ku, *d_kl, *d_vu, *d_vl, *d_ks, *d_kz, *d_vs, *d_vz;
  const size_t code_bytes = (size_t)T2 * 128, meta_bytes = (size_t)T2 * 2;
  CHECK(hip_malloc(&d_ku, code_bytes) == 0 && hip_malloc(&d_kl, code_bytes) == 0);
  CHECK(hip_malloc(&d_vu, code_bytes) == 0 && hip_malloc(&d_vl, code_bytes) == 0);
  CHECK(hip_malloc(&d_ks, meta_bytes) == 0 && hip_malloc(&d_kz, meta_bytes) == 0);
  CHECK(hip_malloc(&d_vs, meta_bytes) == 0 && hip_malloc(&d_vz, meta_bytes) == 0);
  CHECK(export_codes(&c, B - 1, Hkv - 1, T2, d_ku, d_kl, d_ks, d_kz, d_vu, d_vl, d_vs, d_vz, NULL) == QS_OK);
  CHECK(hip_sync() == 0);
  uint8_t *got = malloc(code_bytes);
  CHECK(got != NULL);
  const struct { void *dev; const void *ref; size_t bytes; const char *name; } cmp[] = {
      {d_ku, ku, code_bytes, "ku"}, {d_kl, kl, code_bytes, "kl"}, {d_vu, vu, code_bytes, "vu"}, {d_vl, vl, code_bytes, "vl"},
      {d_ks, ks, meta_bytes, "ks"}, {d_kz, kz, meta_bytes, "kz"}, {d_vs, vs, meta_bytes, "vs"}, {d_vz, vz, meta_bytes, "vz"}};
  for (size_t i = 0; i < sizeof cmp / sizeof cmp[0]; ++i) {
    CHECK(hip_memcpy(got, cmp[i].dev, cmp[i].bytes, D2H) == 0);
    if (memcmp(got, cmp[i].ref, cmp[i].bytes) != 0) {
      fprintf(stderr, "%s differs from the oracle\n", cmp[i].name);
      return 1;
    }
  }
  void *all[] = {c.upper, c.lower, c.k_buf, c.v_buf, k_src, v_src, q_dev, out_dev, ws, d_ku, d_kl, d_vu, d_vl, d_ks, d_kz, d_vs, d_vz};
  for (size_t i = 0; i < sizeof all / sizeof all[0]; ++i) CHECK(hip_free(all[i]) == 0);
  puts("ok");
  return 0;
}
