// C ABI of libquantspec: argument validation, split planning and kernel launches.
// All validation happens before the first HIP call, so error paths can be exercised without a GPU.
#include <algorithm>
#include <atomic>

#include "qs_internal.h"

namespace qs {
namespace {

constexpr int kVersion = 210;   // 0.2.1
constexpr int kDefaultCUs = 256;
// resident chunk waves per compute unit the split planner aims for: one wave per SIMD, two for the draft call
// of 2 - 8 query rows per kv-head (see make_plan)
constexpr int kWavesPerCUSingle = 4;
constexpr int kWavesPerCUPaired = kCuWaves;
constexpr int kMinBufSplits = 8;   // a decode-time buffer (2G + gamma + 1 tokens) always gets its 64-token chunks

constexpr int kMaxDevices = 64;
std::atomic<int> g_cu_count[kMaxDevices];   // compute units of each device, read once (0: not read yet)

// Compute units of the current device.
int device_cu_count() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return kDefaultCUs;
  int n = g_cu_count[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  hipDeviceProp_t prop;
  n = kDefaultCUs;
  if (hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0) n = prop.multiProcessorCount;
  g_cu_count[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Compute units to plan for: the caller's figure, else those of the current device.
int cu_count(const qs_cache* c) { return c->compute_units > 0 ? c->compute_units : device_cu_count(); }

// Split-K partials of qs_attn_static: one array per device, part of the library's code object, so a
// caller that must not allocate needs no workspace of its own.  In host code the array's name only
// stands for the symbol; its address on a device comes from hipGetSymbolAddress() with that device
// current, once, and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[QS_STATIC_WS_BYTES];
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QS_ERR_HIP;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return QS_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // two threads racing here store the same address
  }
  *out = ptr;
  return QS_OK;
}

// head_dim in {64, 128, 256}, group in {32, 64, 128}, whole groups per token row
bool shape_built(int d, int g) {
  return (d == 64 || d == 128 || d == 256) && (g == 32 || g == 64 || g == 128) && d % g == 0;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_shape(const qs_cache* c) {
  if (c == nullptr) return QS_ERR_NULL;
  if (c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->n_q_heads % c->n_kv_heads != 0)
    return QS_ERR_SHAPE;
  if (c->q_cap < 0 || c->q_cap % kG != 0 || c->buf_cap <= 0) return QS_ERR_SHAPE;
  if (c->group_table != nullptr && c->pool_groups <= 0) return QS_ERR_SHAPE;
  if (c->compute_units < 0 || c->compute_units > 65536 || (c->flags & ~(uint32_t)QS_FLAG_FIXED_RANGES) != 0)
    return QS_ERR_RANGE;
  if (!shape_built(c->head_dim, c->group) || c->batch > QS_MAX_BATCH) return QS_ERR_UNSUPPORTED;
  return QS_OK;
}

bool tuned_shape(const qs_cache* c) { return c->head_dim == kD && c->group == kG; }

int validate_cache(const qs_cache* c) {
  int rc = validate_shape(c);
  if (rc != QS_OK) return rc;
  const void* ptrs[] = {c->k_buf, c->v_buf, c->upper, c->lower};
  // a cache without a quantized region (q_cap == 0, everything in the fp16 buffer) needs no planes
  for (int i = 0; i < (c->q_cap > 0 ? 4 : 2); ++i)
    if (ptrs[i] == nullptr) return QS_ERR_NULL;
  if (c->n_quant == nullptr || c->n_buf == nullptr) return QS_ERR_NULL;
  for (const void* p : ptrs)
    if (!aligned16(p)) return QS_ERR_ALIGN;
  for (int b = 0; b < c->batch; ++b) {
    if (c->n_quant[b] < 0 || c->n_quant[b] > c->q_cap || c->n_quant[b] % c->group != 0) return QS_ERR_RANGE;
    if (c->n_buf[b] < 0 || c->n_buf[b] > c->buf_cap) return QS_ERR_RANGE;
  }
  return QS_OK;
}

// Number of chunks per unit.  The quantized region is cut so that about kWavesPerCUSingle (or Paired) waves per
// compute unit are resident; the buffer is cut into 64-token chunks, or, when it is so long that
// these would exceed that budget too, into as many equal chunks as the budget allows.  Depends on
// the descriptor (shapes, compute units, flags) and on the given maximum lengths only.
struct Plan {
  int n_split_q, n_split_b;
  int cu_wgs;   // > 0: workgroups of eight waves per unit, groups drawn dynamically (n_split_q = 8 * cu_wgs)
  int ws_splits;   // partial slots per query row to size the workspace for: covers either way of dealing out
};

Plan make_plan(const qs_cache* c, int nq, int max_quant, int max_buf, bool verify) {
  const int units = c->batch * c->n_kv_heads;
  const int groups = max_quant / kG;
  const int n_rows = nq * (c->n_q_heads / c->n_kv_heads);
  // One wave per SIMD, each on a fixed range, is what the one-tile kernels run best as - measured in the steady
  // state of a decode cycle at the power limit: one query row per kv-head at 128k context 89.8 us against 91.0 us
  // of two waves per SIMD dealt through a queue, the 5-row verify call 169.4 against 173.5 us, at 32k 28.7 / 53.3
  // against 31.2 / 54.5 us - with two exceptions that keep two waves per SIMD and the queue: the draft call
  // of 2 - 8 rows (grouped queries: 92.9 against 101.5 us at 128k, 4 rows) and the draft call of one row over a
  // paged cache (92.7 against 96.2 us; its verify call: 169.6 us with one wave per SIMD, 173.8 with two).
  const bool paired = !verify && n_rows <= 8 && (n_rows >= 2 || c->group_table != nullptr);
  const int wpc = paired ? kWavesPerCUPaired : kWavesPerCUSingle;
  // never more long chunks than resident slots: a chunk that starts late doubles the launch time
  const int want = std::max(1, cu_count(c) * wpc / units);
  Plan p;
  if (!tuned_shape(c)) {   // one-wave workgroups over ranges of 32-token blocks, fixed ranges only
    const int blocks = max_quant / kBlkTok;
    // One-wave workgroups per compute unit, all row batches (grid.z) of a range counted.  Measured on 32 kv-heads x
    // 32k tokens, 1 / 4 / 5 / 20 rows per kv-head, in workgroups per compute unit: fewer, longer ranges often beat
    // filling every slot the registers allow (the waves of a SIMD do not advance at the same pace).
    //   head_dim 64:  12 is within 2 % of the best everywhere (8 - 16 resident);
    //   head_dim 128: 8 (two per SIMD); the verify call of up to 16 rows 4 (49 vs 53 us at groups of 64);
    //   head_dim 256: 4 (one per SIMD); the single-row kernel of the draft call has room for two, which pays
    //                 with groups of 32, where a wave's step is long (64 vs 73 us; 61 vs 58 us with groups of 64,
    //                 57 vs 52 us with 128).
    const int row_batches = c->head_dim == 256 ? (n_rows + 15) / 16 : (n_rows + 31) / 32;
    const int per_cu = c->head_dim == 64    ? 12
                       : c->head_dim == 128 ? (verify && n_rows <= 16 ? 4 : 8)
                                            : (!verify && n_rows == 1 && c->group == 32 ? 8 : 4);
    const int want_plain = std::max(1, cu_count(c) * per_cu / (units * row_batches));
    p.n_split_q = std::max(1, std::min(want_plain, blocks));
    p.n_split_b = std::max(1, std::min((max_buf + kBufSplitTok - 1) / kBufSplitTok, std::max(want_plain, kMinBufSplits)));
    p.cu_wgs = 0;
    p.ws_splits = p.n_split_q + p.n_split_b;
    return p;
  }
  p.n_split_q = std::max(1, std::min(want, groups));
  // the buffer: 64-token chunks while they fit a budget of resident waves, longer ones beyond.  A long
  // full-precision buffer (a cache without a quantized region) streams best with two waves per SIMD where
  // the kernel's registers allow them: 128k tokens x 32 heads 370 us, 392 us with one.
  const int want_buf = std::max(1, cu_count(c) * (n_rows <= 8 ? kWavesPerCUPaired : kWavesPerCUSingle) / units);
  p.n_split_b = std::max(1, std::min((max_buf + kBufSplitTok - 1) / kBufSplitTok, std::max(want_buf, kMinBufSplits)));
  // Two waves per SIMD do not advance at the same pace (the older one wins the issue conflicts), so
  // where two are wanted they run as one eight-wave workgroup per compute unit whose waves share their
  // groups through a queue - when every wave still gets a group and the workgroup's share of the
  // buffer chunks fits its transpose tiles.
  p.cu_wgs = 0;
  p.ws_splits = p.n_split_q + p.n_split_b;
  const int wgs = want / kCuWaves;
  if (paired && (c->flags & QS_FLAG_FIXED_RANGES) == 0 && wgs >= 1 &&
      groups >= kCuWaves * wgs && p.n_split_b <= kCuBufItems * wgs) {
    p.cu_wgs = wgs;
    p.n_split_q = kCuWaves * wgs;
  }
  return p;
}

// dry_run: validate everything but the workspace and launch nothing.
int attn_common(const qs_cache* c, const void* q, int32_t nq, void* out, float sm_scale, void* workspace,
                size_t workspace_bytes, float* lse, void* stream, bool verify, bool dry_run = false) {
  int rc = validate_cache(c);
  if (rc != QS_OK) return rc;
  if (q == nullptr || out == nullptr) return QS_ERR_NULL;
  if (nq < 1 || nq > QS_MAX_NQ) return QS_ERR_UNSUPPORTED;
  if (!(sm_scale > 0.0f) || !(sm_scale < 3.0e38f)) return QS_ERR_RANGE;   // the kernels rely on a positive, finite scale
  if (!aligned16(q) || !aligned16(out) || !aligned16(workspace)) return QS_ERR_ALIGN;
  int max_quant = 0, max_buf = 0;
  for (int b = 0; b < c->batch; ++b) {
    if (c->n_buf[b] < nq) return QS_ERR_RANGE;
    max_quant = std::max(max_quant, c->n_quant[b]);
    max_buf = std::max(max_buf, c->n_buf[b]);
  }
  if (dry_run) return QS_OK;
  if (workspace == nullptr || workspace_bytes < qs_workspace_bytes(c, nq)) return QS_ERR_WORKSPACE;

  const Plan p = make_plan(c, nq, max_quant, max_buf, verify);
  const int n_split = p.n_split_q + p.n_split_b;
  const int64_t rows_total = (int64_t)c->batch * nq * c->n_q_heads;

  AttnArgs a;
  a.head_dim = c->head_dim;
  a.group = c->group;
  a.upper = static_cast<const uint8_t*>(c->upper);
  a.lower = static_cast<const uint8_t*>(c->lower);
  a.group_table = c->group_table;
  a.k_buf = static_cast<const _Float16*>(c->k_buf);
  a.v_buf = static_cast<const _Float16*>(c->v_buf);
  a.q = static_cast<const _Float16*>(q);
  a.ws_o = static_cast<float*>(workspace);
  a.ws_ml = a.ws_o + rows_total * n_split * c->head_dim;
  a.n_q_heads = c->n_q_heads;
  a.n_kv_heads = c->n_kv_heads;
  a.rep = c->n_q_heads / c->n_kv_heads;
  a.nq = nq;
  a.q_cap = c->q_cap;
  a.buf_cap = c->buf_cap;
  a.n_split_q = p.n_split_q;
  a.n_split_b = p.n_split_b;
  a.cu_wgs = p.cu_wgs;
  a.n_rows = nq * a.rep;
  a.c0 = sm_scale * 1.4426950408889634f;
  for (int b = 0; b < QS_MAX_BATCH; ++b) {
    a.len.n_quant[b] = b < c->batch ? c->n_quant[b] : 0;
    a.len.n_buf[b] = b < c->batch ? c->n_buf[b] : 0;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (launch_attn(a, c->batch, verify, s) != hipSuccess) return QS_ERR_HIP;

  MergeArgs m;
  m.head_dim = c->head_dim;
  m.ws_o = a.ws_o;
  m.ws_ml = a.ws_ml;
  m.out = static_cast<_Float16*>(out);
  m.lse = lse;
  m.n_split = n_split;
  if (launch_merge(m, (int)rows_total, s) != hipSuccess) return QS_ERR_HIP;
  return QS_OK;
}

int quantize_common(const qs_cache* c, const _Float16* k_src, const _Float16* v_src, int64_t src_stride,
                    int32_t n_tokens, bool move_buffer, hipStream_t s) {
  FlushArgs f;
  f.head_dim = c->head_dim;
  f.group = c->group;
  f.k_src = k_src;
  f.v_src = v_src;
  f.src_stride = src_stride;
  f.upper = static_cast<uint8_t*>(c->upper);
  f.lower = static_cast<uint8_t*>(c->lower);
  f.group_table = c->group_table;
  f.n_kv_heads = c->n_kv_heads;
  f.q_cap = c->q_cap;
  f.n_groups = n_tokens / c->group;
  f.k_move = move_buffer ? static_cast<_Float16*>(c->k_buf) : nullptr;
  f.v_move = move_buffer ? static_cast<_Float16*>(c->v_buf) : nullptr;
  for (int b = 0; b < QS_MAX_BATCH; ++b) {
    f.n_quant[b] = b < c->batch ? c->n_quant[b] : 0;
    f.n_buf[b] = b < c->batch ? c->n_buf[b] : 0;
  }
  return launch_flush(f, c->batch, s) == hipSuccess ? QS_OK : QS_ERR_HIP;
}

// 4-bit weight layers: the sizes the kernels are built for (the sums of x per group of one launch live in LDS)
constexpr int kW4MaxIn = 32768;
int w4_args(const qs_w4* l, W4Args& a) {
  if (l == nullptr || l->packed == nullptr) return QS_ERR_NULL;
  if (l->n_out <= 0 || l->n_in <= 0 || l->n_out % 16 != 0 || l->n_in % QS_W4_GROUP != 0 || l->n_in > kW4MaxIn)
    return QS_ERR_SHAPE;
  if (!aligned16(l->packed)) return QS_ERR_ALIGN;
  a.packed = static_cast<uint8_t*>(l->packed);
  a.n_out = l->n_out;
  a.n_in = l->n_in;
  return QS_OK;
}

}  // namespace
}  // namespace qs

using namespace qs;

extern "C" {

int qs_version(void) { return kVersion; }

const char* qs_strerror(int code) {
  switch (code) {
    case QS_OK: return "ok";
    case QS_ERR_NULL: return "a required pointer is NULL";
    case QS_ERR_SHAPE: return "inconsistent batch / head counts / capacities";
    case QS_ERR_UNSUPPORTED: return "unsupported configuration (head_dim 64/128/256, group 32/64/128 dividing head_dim, batch <= 256, nq <= 16)";
    case QS_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case QS_ERR_RANGE: return "a length, count or flag is out of range (lengths: within capacity, multiples of the group size)";
    case QS_ERR_WORKSPACE: return "workspace is missing or smaller than qs_workspace_bytes(), or (qs_attn_static) that size exceeds QS_STATIC_WS_BYTES";
    case QS_ERR_HIP: return "a HIP runtime call failed";
    default: return "unknown status code";
  }
}

size_t qs_workspace_bytes(const qs_cache* c, int32_t nq) {
  if (validate_shape(c) != QS_OK || nq < 1 || nq > QS_MAX_NQ) return 0;
  // the larger of the two calls' plans at full capacity
  const int splits = std::max(make_plan(c, nq, c->q_cap, c->buf_cap, false).ws_splits,
                              make_plan(c, nq, c->q_cap, c->buf_cap, true).ws_splits);
  const size_t rows_total = (size_t)c->batch * nq * c->n_q_heads;
  return rows_total * (size_t)splits * (c->head_dim + 2) * sizeof(float);
}

int qs_quantize_flush(const qs_cache* c, int32_t n_tokens, void* stream) {
  int rc = validate_cache(c);
  if (rc != QS_OK) return rc;
  if (n_tokens < 0 || n_tokens % c->group != 0) return QS_ERR_RANGE;
  for (int b = 0; b < c->batch; ++b)
    if (n_tokens > c->n_buf[b] || c->n_quant[b] + n_tokens > c->q_cap) return QS_ERR_RANGE;
  if (n_tokens == 0) return QS_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // one group: the flush kernel moves the rest of the buffer itself; more: a second kernel does
  const bool fused = flush_moves_buffer(c->head_dim, c->group, n_tokens / c->group, c->batch * c->n_kv_heads);
  rc = quantize_common(c, static_cast<const _Float16*>(c->k_buf), static_cast<const _Float16*>(c->v_buf),
                       c->buf_cap, n_tokens, fused, s);
  if (rc != QS_OK || fused) return rc;
  ShiftArgs sh;
  sh.head_dim = c->head_dim;
  sh.k_buf = static_cast<_Float16*>(c->k_buf);
  sh.v_buf = static_cast<_Float16*>(c->v_buf);
  sh.n_kv_heads = c->n_kv_heads;
  sh.buf_cap = c->buf_cap;
  sh.n_tokens = n_tokens;
  bool any = false;
  for (int b = 0; b < QS_MAX_BATCH; ++b) {
    sh.n_buf[b] = b < c->batch ? c->n_buf[b] : 0;
    any |= b < c->batch && c->n_buf[b] > n_tokens;
  }
  if (any && launch_shift(sh, c->batch, s) != hipSuccess) return QS_ERR_HIP;
  return QS_OK;
}

int qs_quantize_prefill(const qs_cache* c, const void* k_src, const void* v_src, int64_t src_stride_tokens,
                        int32_t n_tokens, void* stream) {
  int rc = validate_cache(c);
  if (rc != QS_OK) return rc;
  if (k_src == nullptr || v_src == nullptr) return QS_ERR_NULL;
  if (!aligned16(k_src) || !aligned16(v_src)) return QS_ERR_ALIGN;
  if (n_tokens < 0 || n_tokens % c->group != 0 || src_stride_tokens < n_tokens) return QS_ERR_RANGE;
  for (int b = 0; b < c->batch; ++b)
    if (c->n_quant[b] + n_tokens > c->q_cap) return QS_ERR_RANGE;
  if (n_tokens == 0) return QS_OK;
  return quantize_common(c, static_cast<const _Float16*>(k_src), static_cast<const _Float16*>(v_src),
                         src_stride_tokens, n_tokens, false, static_cast<hipStream_t>(stream));
}

int qs_append(const qs_cache* c, const void* k_new, const void* v_new, int32_t n_new, void* stream) {
  int rc = validate_cache(c);
  if (rc != QS_OK) return rc;
  if (k_new == nullptr || v_new == nullptr) return QS_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new)) return QS_ERR_ALIGN;
  if (n_new < 0) return QS_ERR_RANGE;
  for (int b = 0; b < c->batch; ++b)
    if (c->n_buf[b] + n_new > c->buf_cap) return QS_ERR_RANGE;
  if (n_new == 0) return QS_OK;
  AppendArgs a;
  a.head_dim = c->head_dim;
  a.k_new = static_cast<const _Float16*>(k_new);
  a.v_new = static_cast<const _Float16*>(v_new);
  a.k_buf = static_cast<_Float16*>(c->k_buf);
  a.v_buf = static_cast<_Float16*>(c->v_buf);
  a.n_kv_heads = c->n_kv_heads;
  a.buf_cap = c->buf_cap;
  a.n_new = n_new;
  for (int b = 0; b < QS_MAX_BATCH; ++b) a.n_buf[b] = b < c->batch ? c->n_buf[b] : 0;
  return launch_append(a, c->batch, static_cast<hipStream_t>(stream)) == hipSuccess ? QS_OK : QS_ERR_HIP;
}

int qs_attn_draft(const qs_cache* c, const void* q, void* out, float sm_scale, void* workspace,
                  size_t workspace_bytes, float* lse, void* stream) {
  return attn_common(c, q, 1, out, sm_scale, workspace, workspace_bytes, lse, stream, false);
}

int qs_attn_verify(const qs_cache* c, const void* q, int32_t nq, void* out, float sm_scale, void* workspace,
                   size_t workspace_bytes, float* lse, void* stream) {
  return attn_common(c, q, nq, out, sm_scale, workspace, workspace_bytes, lse, stream, true);
}

int qs_attn_static(const qs_cache* c, const void* q, int32_t nq, int32_t verify, void* out, float sm_scale, float* lse,
                   void* stream) {
  if (verify != 0 && verify != 1) return QS_ERR_RANGE;
  if (!verify && nq != 1) return QS_ERR_UNSUPPORTED;
  const size_t need = qs_workspace_bytes(c, nq);   // 0 for a descriptor that attn_common rejects anyway
  if (need > QS_STATIC_WS_BYTES) return QS_ERR_WORKSPACE;
  // everything else is checked before the first HIP call: a dry run against a stand-in address
  int rc = attn_common(c, q, nq, out, sm_scale, nullptr, 0, lse, stream, verify != 0, /*dry_run=*/true);
  if (rc != QS_OK) return rc;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != QS_OK) return rc;
  return attn_common(c, q, nq, out, sm_scale, ws, QS_STATIC_WS_BYTES, lse, stream, verify != 0);
}

int qs_export_codes(const qs_cache* c, int32_t b, int32_t kv_head, int32_t n_tokens, void* k_u, void* k_l,
                    void* k_s, void* k_z, void* v_u, void* v_l, void* v_s, void* v_z, void* stream) {
  int rc = validate_cache(c);
  if (rc != QS_OK) return rc;
  if (b < 0 || b >= c->batch || kv_head < 0 || kv_head >= c->n_kv_heads) return QS_ERR_RANGE;
  if (n_tokens < 0 || n_tokens % c->group != 0 || n_tokens > c->q_cap) return QS_ERR_RANGE;
  const int64_t unit = (int64_t)b * c->n_kv_heads + kv_head;
  ExportArgs e;
  e.head_dim = c->head_dim;
  e.group = c->group;
  e.upper = static_cast<const uint8_t*>(c->upper);
  e.lower = static_cast<const uint8_t*>(c->lower);
  e.group_table = c->group_table;
  e.unit = (int32_t)unit;
  e.q_cap = c->q_cap;
  e.k_s = static_cast<_Float16*>(k_s);
  e.k_z = static_cast<_Float16*>(k_z);
  e.k_u = static_cast<uint8_t*>(k_u);
  e.k_l = static_cast<int8_t*>(k_l);
  e.v_u = static_cast<uint8_t*>(v_u);
  e.v_l = static_cast<int8_t*>(v_l);
  e.v_s = static_cast<_Float16*>(v_s);
  e.v_z = static_cast<_Float16*>(v_z);
  e.n_tokens = n_tokens;
  return launch_export(e, static_cast<hipStream_t>(stream)) == hipSuccess ? QS_OK : QS_ERR_HIP;
}

size_t qs_w4_bytes(int32_t n_out, int32_t n_in) {
  if (n_out <= 0 || n_in <= 0 || n_out % 16 != 0 || n_in % QS_W4_GROUP != 0 || n_in > kW4MaxIn) return 0;
  return (size_t)(n_out / 16) * (size_t)(n_in / QS_W4_GROUP) * kW4Block;
}

int qs_w4_quantize(const qs_w4* l, const void* w, void* stream) {
  W4Args a{};
  int rc = w4_args(l, a);
  if (rc != QS_OK) return rc;
  if (w == nullptr) return QS_ERR_NULL;
  if (!aligned16(w)) return QS_ERR_ALIGN;
  a.w = static_cast<const _Float16*>(w);
  return launch_w4_quantize(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QS_OK : QS_ERR_HIP;
}

int qs_w4_linear(const qs_w4* l, const void* x, int32_t m, void* y, void* stream) {
  W4Args a{};
  int rc = w4_args(l, a);
  if (rc != QS_OK) return rc;
  if (x == nullptr || y == nullptr) return QS_ERR_NULL;
  if (!aligned16(x) || !aligned16(y)) return QS_ERR_ALIGN;
  if (m < 1 || m > QS_W4_MAX_ROWS) return QS_ERR_SHAPE;
  a.x = static_cast<const _Float16*>(x);
  a.y = static_cast<_Float16*>(y);
  a.m = m;
  return launch_w4_linear(a, device_cu_count(), static_cast<hipStream_t>(stream)) == hipSuccess ? QS_OK : QS_ERR_HIP;
}

int qs_w4_export(const qs_w4* l, void* codes, void* scale, void* zero, void* stream) {
  W4Args a{};
  int rc = w4_args(l, a);
  if (rc != QS_OK) return rc;
  a.codes = static_cast<uint8_t*>(codes);
  a.scale = static_cast<_Float16*>(scale);
  a.zero = static_cast<_Float16*>(zero);
  return launch_w4_export(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QS_OK : QS_ERR_HIP;
}

}  // extern "C"
