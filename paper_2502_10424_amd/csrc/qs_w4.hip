// The draft model's linear layers with 4-bit weights (abstract; Section 4): y = x W_hat^T for a few rows
// of x (the decode step of the draft model: one row per sequence).  Bound by the HBM stream of the codes.
//
// The weights lie in blocks of 16 output rows x 128 input channels (quantspec.h): 1 KB of codes in the
// order the lanes of a wave take them as matrix-core operands, and, in a region of their own, the 16 rows'
// scales and zeros.  A code
// c, zero-extended to 16 bits, is the fp16 subnormal c * 2^-24 and goes to the matrix cores as it is, x as
// it is: products exact, sums in binary32.  For one block
//     sum_k x_k (c_k S + Z) = S * (sum_k c_k x_k) + Z * (sum_k x_k):
// the first sum is four MFMA steps, the second depends on x alone and is formed once per launch.
//
// A tile of 16 output rows gets as many waves (W = 1 .. 16) as let all tiles be resident at once: a layer of a
// few tens of MB is over in microseconds, and a second round of workgroups would pay the whole chain of
// latencies again.  Wave w of the W takes the blocks g = w, w + W, ... of the tile's row of blocks (contiguous
// in memory, so the waves of a tile stream one run), with the words of the next kAhead of its blocks requested
// ahead - one 1 KB load per block and wave: the scales and zeros of the workgroup's tiles are staged in LDS once,
// with wide loads (fetched per block, as two small loads beside the wide one, they cost 15 - 25 % of the call
// time: a load instruction occupies the memory pipeline by its lanes, not by its bytes); the W partial sums
// meet in LDS in a fixed order (deterministic).  Tiles with few waves
// each share a workgroup of up to eight waves, so that one copy of x in LDS serves several of them.
// Every step issues the same loads - a block past the end is asked for through buffer resources of no bytes,
// which return zero without touching memory - so the wait for a block's words is a count, not a drain.
// x is staged in LDS once per workgroup when it fits (XLDS: the decode step's one or few rows); otherwise a
// lane's pieces of x travel with the block's words.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "qs_internal.h"

namespace qs {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMaxWaves = 16, kAhead = 2;
constexpr int kGroupedWaves = 8;           // tiles with fewer waves each share a workgroup of up to this many
constexpr int kBufferWord3 = 0x00020000;   // raw 32-bit elements (gfx9 family)
constexpr int kAuxStream = 2;              // non-temporal: the weights are read once per launch
constexpr size_t kW4XLdsBytes = 65536;     // x is staged in LDS up to this size (one row of the longest x the library takes)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t resource(const void* base, uint32_t bytes) {
  // the address is the same in every lane; saying so keeps the descriptor in scalar registers
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<uint8_t*>((hi << 32) | lo), 0, (int)bytes, kBufferWord3);
}

// Eight 4-bit codes of a word -> eight fp16 subnormals c * 2^-24; element i comes from nibble (i&1)*4 + (i>>1).
__device__ __forceinline__ half8 code_operand(uint32_t w) {
  u32x4 r;
  r[0] = w & 0x000F000Fu;
  r[1] = (w >> 4) & 0x000F000Fu;
  r[2] = (w >> 8) & 0x000F000Fu;
  r[3] = (w >> 12) & 0x000F000Fu;
  return __builtin_bit_cast(half8, r);
}

template <bool XLDS>
__global__ __launch_bounds__(64 * kMaxWaves) void w4_linear_kernel(W4Args a) {
  // sum of x over each group of 128 inputs, [group][row of x]; the waves' partial results; the scales and zeros of
  // the workgroup's tiles; x itself (XLDS)
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int groups = a.n_in / 128;
  float* xsum = reinterpret_cast<float*>(lds);
  float4v* red = reinterpret_cast<float4v*>(lds + (((size_t)groups * a.m * sizeof(float) + 15) & ~(size_t)15));
  const int tid = threadIdx.x, lane = tid & 63, n_waves = blockDim.x >> 6, n_threads = blockDim.x;
  // the same in every lane of a wave; saying so keeps block numbers and resource descriptors in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wpt = a.waves_per_tile, tile_local = wave / wpt, w = wave % wpt, tiles = a.n_out / 16;
  uint8_t* meta_lds = reinterpret_cast<uint8_t*>(red + n_waves * 64);   // [tile of the workgroup][group][64 bytes]
  uint8_t* x_lds = meta_lds + (size_t)(n_waves / wpt) * groups * kW4Meta;
  const int rho = lane & 15, q4 = lane >> 4;   // lane = 16 * q4 + rho: output rows 4 q4 .. 4 q4 + 3, row rho of x
  const int T = blockIdx.x * (n_waves / wpt) + tile_local;
  const bool active = T < tiles;   // the last workgroup may have waves without a tile: they only help with x

  struct Slot {
    u32x4 w;                  // code words of the four matrix-core steps
    u32x4 sz;                 // S (four halves), then Z of output rows 4 q4 .. 4 q4 + 3
    u32x4 x[4];               // x[rho][128 g + 32 s + 8 q4 ..], s < 4
    float xs;                 // sum of x[rho] over the block's 128 inputs (XLDS: read ahead like x)
  };
  const uint8_t* row_of_blocks = a.packed + (int64_t)min(T, tiles - 1) * groups * kW4Codes;
  const uint32_t x_bytes = (uint32_t)a.m * (uint32_t)a.n_in * 2u;
  // One resource for the tile's row of blocks (none of its bytes for a wave without a tile): a block is an offset
  // into it (in the lanes' offsets, which the range check covers), and a block past the end of the row lies past
  // the end of the resource.
  const __amdgpu_buffer_rsrc_t rw = resource(row_of_blocks, active ? (uint32_t)groups * kW4Codes : 0u);
  const __amdgpu_buffer_rsrc_t rx = resource(a.x, active ? x_bytes : 0u);   // rows of x past m read as zero
  auto request = [&](Slot& sl, int g) __attribute__((always_inline)) {
    sl.w = __builtin_amdgcn_raw_buffer_load_b128(rw, g * kW4Codes + lane * 16, 0, kAuxStream);
    if constexpr (!XLDS) {   // a block past the end: any block's inputs, against codes, scales and zeros that read as zero
#pragma unroll
      for (int s = 0; s < 4; ++s)
        sl.x[s] = __builtin_amdgcn_raw_buffer_load_b128(rx, (rho * a.n_in + 128 * min(g, groups - 1) + 32 * s + 8 * q4) * 2, 0, 0);
    }
  };
  // What a block needs from LDS - its scales and zeros, and (XLDS) its inputs and their sum - is read when the
  // block's words are requested, not when they have arrived: the wait for the words then hides the LDS round
  // trip.  Columns past m take the last row's numbers: their results are never stored.
  auto from_lds_ahead = [&](Slot& sl, int g) __attribute__((always_inline)) {
    const int gc = min(g, groups - 1), row = min(rho, a.m - 1);
    sl.sz = *reinterpret_cast<const u32x4*>(meta_lds + ((tile_local * groups + gc) * 4 + q4) * 16);
    if constexpr (XLDS) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
        sl.x[s] = *reinterpret_cast<const u32x4*>(x_lds + (row * a.n_in + 128 * gc + 32 * s + 8 * q4) * 2);
      sl.xs = xsum[gc * a.m + row];
    }
  };
  Slot slot[kAhead];
#pragma unroll
  for (int k = 0; k < kAhead; ++k) request(slot[k], w + wpt * k);

  {   // the scales and zeros of the workgroup's tiles -> LDS: one contiguous run, 16 bytes per thread and piece
    const int tiles_here = min(n_waves / wpt, tiles - (int)blockIdx.x * (n_waves / wpt));
    const int pieces = tiles_here * groups * (kW4Meta / 16);
    const __amdgpu_buffer_rsrc_t rm = resource(a.packed + w4_meta_base(a.n_out, a.n_in) +
                                               (int64_t)blockIdx.x * (n_waves / wpt) * groups * kW4Meta, (uint32_t)pieces * 16u);
    for (int base = tid; base < pieces; base += 4 * n_threads) {
      u32x4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = __builtin_amdgcn_raw_buffer_load_b128(rm, (base + j * n_threads) * 16, 0, 0);   // past the end: zero
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (base + j * n_threads < pieces) reinterpret_cast<u32x4*>(meta_lds)[base + j * n_threads] = v[j];
    }
    if constexpr (!XLDS) __syncthreads();   // (XLDS: the barrier after the staging of x serves both)
  }
  if constexpr (XLDS) {   // x -> LDS, 16 bytes per thread and piece, eight pieces requested before the first is stored
    const int pieces = a.m * a.n_in / 8;
    const __amdgpu_buffer_rsrc_t rs = resource(a.x, x_bytes);   // every wave stages, also one without a tile
    for (int base = tid; base < pieces; base += 8 * n_threads) {
      u32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, (base + j * n_threads) * 16, 0, 0);   // past the end: zero
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (base + j * n_threads < pieces) reinterpret_cast<u32x4*>(x_lds)[base + j * n_threads] = v[j];
    }
    __syncthreads();
  }

  // ---- sums of x per group: 16 lanes to a (group, row) pair, eight inputs each ----
  {
    const int sub = tid & 15;
    for (int item = tid >> 4; item < groups * a.m; item += n_threads >> 4) {
      const int g = item / a.m, row = item % a.m;
      const int at = row * a.n_in + 128 * g + 8 * sub;
      const half8 v = XLDS ? *reinterpret_cast<const half8*>(x_lds + 2 * at) : *reinterpret_cast<const half8*>(a.x + at);
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) sum += (float)v[i];
#pragma unroll
      for (int m = 1; m < 16; m <<= 1) sum += __shfl_xor(sum, m);
      if (sub == 0) xsum[g * a.m + row] = sum;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kAhead; ++k) from_lds_ahead(slot[k], w + wpt * k);

  float4v out_s = {0.f, 0.f, 0.f, 0.f}, out_z = {0.f, 0.f, 0.f, 0.f};   // sum of S * (codes . x) * 2^-24, and of Z * sum x
  auto consume = [&](const Slot& sl, int g) __attribute__((always_inline)) {
    // two chains of two steps: a step waits for the matrix cores' result of the one before it in its chain
    float4v acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(sl.w[0]), __builtin_bit_cast(half8, sl.x[0]), acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(sl.w[1]), __builtin_bit_cast(half8, sl.x[1]), acc1, 0, 0, 0);
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(sl.w[2]), __builtin_bit_cast(half8, sl.x[2]), acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand(sl.w[3]), __builtin_bit_cast(half8, sl.x[3]), acc1, 0, 0, 0);
    const float xs = XLDS ? sl.xs : xsum[min(g, groups - 1) * a.m + min(rho, a.m - 1)];
    const half8 sz = __builtin_bit_cast(half8, sl.sz);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      out_s[jj] = __builtin_fmaf(acc0[jj] + acc1[jj], (float)sz[jj], out_s[jj]);
      out_z[jj] = __builtin_fmaf(xs, (float)sz[4 + jj], out_z[jj]);
    }
  };
  for (int g0 = active ? w : groups; g0 < groups; g0 += wpt * kAhead) {
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      if (g0 + wpt * k < groups) consume(slot[k], g0 + wpt * k);   // the requests stay unconditional
      request(slot[k], g0 + wpt * (k + kAhead));
      from_lds_ahead(slot[k], g0 + wpt * (k + kAhead));
    }
  }

  // ---- the waves' partial results, added in the order of the waves ----
  float4v part;
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) part[jj] = __builtin_fmaf(out_s[jj], 16777216.0f, out_z[jj]);
  red[wave * 64 + lane] = part;
  __syncthreads();
  if (w == 0 && active && rho < a.m) {
    float4v y = red[wave * 64 + lane];
    for (int j = 1; j < wpt; ++j) y += red[(wave + j) * 64 + lane];
    half4 h;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) h[jj] = (_Float16)y[jj];
    *reinterpret_cast<half4*>(a.y + (int64_t)rho * a.n_out + 16 * T + 4 * q4) = h;
  }
}

}  // namespace

hipError_t launch_w4_linear(const W4Args& a, int compute_units, hipStream_t s) {
  const int tiles = a.n_out / 16, groups = a.n_in / 128;
  // as many waves per tile as keep every tile resident at once (16 waves per compute unit), at most one per block
  W4Args b = a;
  b.waves_per_tile = std::max(1, std::min({kMaxWaves, groups, compute_units * 16 / tiles}));
  const int tiles_per_wg = std::max(1, std::min(kGroupedWaves / b.waves_per_tile, tiles));
  const int waves = b.waves_per_tile * tiles_per_wg;
  const size_t x_bytes = (size_t)a.m * a.n_in * 2;
  const bool xlds = x_bytes <= kW4XLdsBytes;
  const size_t lds = (((size_t)groups * a.m * sizeof(float) + 15) & ~(size_t)15) + (size_t)waves * 64 * sizeof(float4v) +
                     (size_t)tiles_per_wg * groups * kW4Meta + (xlds ? x_bytes : 0);
  void* kargs[] = {&b};
  const void* kernel = xlds ? reinterpret_cast<const void*>(w4_linear_kernel<true>) : reinterpret_cast<const void*>(w4_linear_kernel<false>);
  return hipLaunchKernel(kernel, dim3((tiles + tiles_per_wg - 1) / tiles_per_wg), dim3(64 * waves), kargs, lds, s);
}

}  // namespace qs
