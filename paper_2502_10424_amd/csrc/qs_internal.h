// Internal declarations shared by the translation units of libquantspec (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "quantspec.h"

namespace qs {

constexpr int kD = 128;            // head_dim
constexpr int kG = 128;            // quantization group size
constexpr int kRowDw = 16;         // 32-bit words per token row of key codes (128 nibbles)
constexpr int kBlkTok = 32;        // tokens per cache block
// Byte offsets inside one 32-token block of the upper array (see quantspec.h) ...
constexpr int kOffK = 0;           // key codes: 32 token rows of 64 bytes
constexpr int kOffV = 2048;        // value codes: one 2 KB tile in operand order
constexpr int kOffVS = 4096;       // value scale, 32 fp16 in tile order
constexpr int kOffVZ = 4160;       // value zero
constexpr int kOffKS = 4224;       // key scale of k-step (block mod 4) of the block's group, 32 fp16
constexpr int kOffKZ = 4288;       // key zero, likewise
constexpr int kUpperBlk = 4352;    // bytes per block of the upper array
// ... and of the lower array: key codes at 0, value codes at 2048
constexpr int kLowerBlk = 4096;
// queue-dealt attention kernel: waves of a workgroup (two per SIMD of a compute unit) and the buffer chunks
// one workgroup can take (one transpose tile each)
constexpr int kCuWaves = 8, kCuBufItems = 4;
constexpr int kBulkGroups = 512;   // from this many (group, unit) pairs on, quantization takes the bulk kernel
constexpr int kBufSplitTok = 64;   // buffer tokens handled by one wave of the attention kernel

// Other shapes than head_dim = group = 128 (head_dim 64 / 128 / 256, group 32 / 64 / 128 with group <=
// head_dim) keep the quantized region in plain order, cut into "superblocks" of 128 tokens (see
// quantspec.h).  Byte offsets inside a 128-token row of the upper array; the lower array holds its codes
// at the same offsets and no metadata.
constexpr int kSuper = 128;
struct ShapeLayout {
  int32_t d, g;
  __host__ __device__ int vg() const { return d / g; }                       // value groups per token
  __host__ __device__ int ks() const { return d / 32; }                      // 32-channel steps of a key row
  // codes: four 32-token blocks per row, each 16 d bytes of key codes, then 16 d bytes of value codes
  __host__ __device__ int off_k(int p) const { return p * 32 * d; }
  __host__ __device__ int off_v(int p) const { return p * 32 * d + 16 * d; }
  // 32-bit word of a key block with channels 32 s + 8 g + i (nibble (i&1)*4 + (i>>1)) of token 16 t + rho, lane = 16 g + rho:
  // a lane's words lie four in a row (one 16-byte load): four key steps of one token tile, or, at head_dim 64, the
  // two steps of both tiles
  __host__ __device__ int k_word(int t, int lane, int s) const {
    return ks() == 2 ? lane * 4 + 2 * t + s : ((t * (ks() / 4) + s / 4) * 64 + lane) * 4 + s % 4;
  }
  // 32-bit word of a value block with channel 16 n + rho of tokens 16 (j >> 2) + 4 g + (j & 3) (nibble (j&1)*4 + (j>>1))
  __host__ __device__ int v_word(int n, int lane) const { return ((n >> 2) * 64 + lane) * 4 + (n & 3); }
  __host__ __device__ int off_vs() const { return 128 * d; }                 // value scale, fp16 [128][vg]
  __host__ __device__ int off_vz() const { return 128 * d + 256 * vg(); }    // value zero
  __host__ __device__ int off_ks() const { return 128 * d + 512 * vg(); }    // key scale, fp16 [128 / g][d]
  __host__ __device__ int off_kz() const { return off_ks() + (kSuper / g) * d * 2; }
  __host__ __device__ int upper_bytes() const { return off_kz() + (kSuper / g) * d * 2; }   // = 128 d + 1024 d / g
  __host__ __device__ int lower_bytes() const { return 128 * d; }
};

// Per-sequence lengths travel inside the kernel arguments.
struct SeqLens {
  int32_t n_quant[QS_MAX_BATCH];
  int32_t n_buf[QS_MAX_BATCH];
};

struct FlushArgs {
  int32_t head_dim, group;   // 128, 128: the blocked layout and its kernels; else the plain layout
  const _Float16* k_src;   // [B][Hkv][src_stride][head_dim]
  const _Float16* v_src;
  int64_t src_stride;      // tokens between consecutive units of the source
  uint8_t *upper, *lower;
  const int32_t* group_table;            // device, [units][q_cap/128], or null: contiguous units
  int32_t n_kv_heads, q_cap, n_groups;   // n_groups = n_tokens / 128
  int32_t n_quant[QS_MAX_BATCH];
  // Buffer move done by the flush kernel itself (one flushed group, source = the buffer): rows
  // [128, n_buf) of k_move / v_move become rows [0, n_buf - 128).  Null: no move.
  _Float16 *k_move, *v_move;
  int32_t n_buf[QS_MAX_BATCH];
};

struct ShiftArgs {
  int32_t head_dim;
  _Float16 *k_buf, *v_buf;
  int32_t n_kv_heads, buf_cap, n_tokens;
  int32_t n_buf[QS_MAX_BATCH];
};

struct AppendArgs {
  int32_t head_dim;
  const _Float16 *k_new, *v_new;   // [B][n_new][Hkv][head_dim]
  _Float16 *k_buf, *v_buf;
  int32_t n_kv_heads, buf_cap, n_new;
  int32_t n_buf[QS_MAX_BATCH];
};

struct ExportArgs {
  int32_t head_dim, group;
  const uint8_t *upper, *lower;
  const int32_t* group_table;     // see FlushArgs
  int32_t unit, q_cap;
  uint8_t *k_u, *v_u;
  int8_t *k_l, *v_l;
  _Float16 *k_s, *k_z, *v_s, *v_z;
  int32_t n_tokens;
};

struct AttnArgs {
  int32_t head_dim, group;
  const uint8_t *upper, *lower;
  const int32_t* group_table;     // see FlushArgs
  const _Float16 *k_buf, *v_buf;
  const _Float16* q;       // [B][nq][Hq][128]
  float* ws_o;             // [rows_total][n_split][128] unnormalised partial outputs
  float* ws_ml;            // [rows_total][n_split][2]   (running max in log2 units, sum)
  int32_t n_q_heads, n_kv_heads, rep, nq, q_cap, buf_cap;
  int32_t n_split_q, n_split_b, n_rows;   // n_rows = nq * rep query rows per unit
  int32_t cu_wgs;          // > 0: eight-wave workgroups per unit that draw groups dynamically (n_split_q = 8 * cu_wgs)
  float c0;                // sm_scale * log2(e)
  SeqLens len;
};

struct MergeArgs {
  int32_t head_dim;
  const float *ws_o, *ws_ml;
  _Float16* out;           // [rows_total][head_dim]
  float* lse;              // [rows_total] or null
  int32_t n_split;
};

// Place, counted in 128-token groups, of logical group g of a unit inside the upper / lower arrays.
template <typename Args>
__device__ __forceinline__ int64_t physical_group(const Args& a, int unit, int g) {
  const int64_t logical = (int64_t)unit * (a.q_cap / kG) + g;
  return a.group_table != nullptr ? (int64_t)a.group_table[logical] : logical;
}

// Launches a kernel that takes one argument struct and returns the status of that launch alone: an
// error that an earlier call of the application left behind on this thread is neither reported nor
// consumed (hipGetLastError() would do both).
template <typename K, typename A>
hipError_t launch(K kernel, dim3 grid, dim3 block, hipStream_t s, A args) {
  void* kargs[] = {&args};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, kargs, 0, s);
}

// True if a flush of n_groups groups of `units` units takes the kernel that can also move the buffer.
bool flush_moves_buffer(int head_dim, int group, int n_groups, int units);
hipError_t launch_flush(const FlushArgs& a, int batch, hipStream_t s);
hipError_t launch_shift(const ShiftArgs& a, int batch, hipStream_t s);
hipError_t launch_export(const ExportArgs& a, hipStream_t s);
hipError_t launch_append(const AppendArgs& a, int batch, hipStream_t s);
hipError_t launch_attn(const AttnArgs& a, int batch, bool verify, hipStream_t s);
hipError_t launch_merge(const MergeArgs& a, int rows_total, hipStream_t s);

// ---- 4-bit weights: blocks of 16 output rows x 128 input channels (see quantspec.h) ----
constexpr int kW4Block = 1088;                   // bytes per block in all
constexpr int kW4Codes = 1024, kW4Meta = 64;     // of which codes (first region of `packed`) and scales / zeros (second region)
// Region of the scales and zeros, and where rows 4a .. 4a+3 of block (T, g) keep theirs in it: S (8 bytes), then Z
__host__ __device__ inline int64_t w4_meta_base(int n_out, int n_in) { return (int64_t)(n_out / 16) * (n_in / 128) * kW4Codes; }
struct W4Args {
  uint8_t* packed;
  int n_out, n_in;
  const _Float16* w;        // quantize: [n_out][n_in]
  const _Float16* x;        // linear: [m][n_in]
  _Float16* y;              // linear: [m][n_out]
  int m;
  int waves_per_tile;       // linear: set by the launcher
  uint8_t* codes;           // export
  _Float16* scale;
  _Float16* zero;
};
hipError_t launch_w4_quantize(const W4Args& a, hipStream_t s);
hipError_t launch_w4_export(const W4Args& a, hipStream_t s);
hipError_t launch_w4_linear(const W4Args& a, int compute_units, hipStream_t s);

}  // namespace qs
