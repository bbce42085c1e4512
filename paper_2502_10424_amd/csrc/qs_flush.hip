// Quantize-on-flush, buffer move and plane export kernels (gfx950).
//
// Encoding (paper Section 4.2): per group, Z = min, S = (max - min)/15 stored as fp16; then with
// the stored S and Z, in binary32 and one rounding per operation (this file is compiled with
// -ffp-contract=off):  C_U = clamp(rne((x - Z)/S), 0, 15);  E_U = x - (C_U*S + Z);
// C_L = clamp(rne(E_U / (S/16)), -8, 7).  Keys are grouped per channel over 128 tokens, values per
// token over the 128 channels (Section 4.3.1).
//
// Every thread owns a few channels of the eight tokens that share one 32-bit word of the value-plane
// tile, so value words are assembled in registers and each plane is written exactly once.
#include <type_traits>

#include "qs_internal.h"

namespace qs {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ half8 ld_half8(const _Float16* p) {
  return *reinterpret_cast<const half8*>(p);
}

// Token (inside a 32-token value tile) that sits at operand position j of lane group g, and the
// nibble of the 32-bit word that holds it.  The attention kernel consumes exactly this order.
__device__ __forceinline__ int tile_token(int g, int j) { return ((j >> 2) << 4) + 4 * g + (j & 3); }
__device__ __forceinline__ int tile_nibble(int j) { return ((j & 1) << 2) + (j >> 1); }

// C_U in [0, 15] and C_L in [-8, 7], kept as floats: codes are packed into plane words with exact
// float arithmetic (see pack4) and converted to integers four at a time.
struct Codes {
  float u, l;
};

// The definition: every operation rounds once, in binary32 (Section 4.2).
__device__ __forceinline__ Codes encode(float x, float s, float z) {
  float t = (x - z) / s;
  float u = fminf(fmaxf(rintf(t), 0.0f), 15.0f);
  float deq = u * s;
  deq = deq + z;
  float e = x - deq;
  float sl = s / 16.0f;
  float l = fminf(fmaxf(rintf(e / sl), -8.0f), 7.0f);
  return Codes{u, l};
}

__device__ __forceinline__ _Float16 make_scale(float mn, float mx) {
  float s = (mx - mn) / 15.0f;
  _Float16 h = (_Float16)s;
  if (h == (_Float16)0.0f) h = (_Float16)1.0f;
  return h;
}

// Same codes as encode() at a fraction of the arithmetic.  Both quotients are first formed with an
// approximate reciprocal r of the group's scale (relative error at most 2^-22): t' = fl((x - z) * r)
// and q' = fl(e * 16r).  A quotient of magnitude below 16 differs from its correctly rounded value by
// less than 2^-17 this way (16 * (2^-22 + 2^-24) for r and the product, 2^-21 for the rounding of the
// exact quotient); larger ones only occur beyond the clamps, where both routes give the end code.  So
// whenever t' and q' both stay at least 2^-16 away from every half-integer, rounding them gives the
// codes of encode().  Everything else is the same operation in both: x - z; C_U*S is exact (4 bits
// times 11), so fma(C_U, S, Z) is fl(fl(C_U*S) + Z); E_U = x - that.  x >= Z makes t' >= 0, so the
// lower clamp of C_U never acts.  Otherwise the element takes encode() itself; on fp16 data that is a
// few elements in ten thousand.
struct GroupScale {
  float s, z, r, rl;
};

__device__ __forceinline__ GroupScale group_scale(float s, float z) {
  GroupScale g;
  g.s = s;
  g.z = z;
  g.r = __builtin_amdgcn_rcpf(s);   // s is a normal binary32 number in [2^-24, 2^14)
  g.rl = 16.0f * g.r;               // exact
  return g;
}

struct FastCodes {
  Codes c;
  float off;   // larger distance of t' and q' from their roundings, in [0, 0.5]
};
constexpr float kTie = 0.5f - 0x1p-16f;

__device__ __forceinline__ FastCodes encode_candidate(float x, const GroupScale& g) {
  const float t = (x - g.z) * g.r;
  const float tr = rintf(t);
  const float u = fminf(tr, 15.0f);
  const float e = x - __builtin_fmaf(u, g.s, g.z);
  const float q = e * g.rl;
  const float qr = rintf(q);
  FastCodes f;
  f.c = Codes{u, __builtin_amdgcn_fmed3f(qr, -8.0f, 7.0f)};
  // both distances are at most 0.5, so the median of them and 1 is the larger one
  f.off = __builtin_amdgcn_fmed3f(fabsf(t - tr), fabsf(q - qr), 1.0f);
  return f;
}

__device__ __forceinline__ Codes encode_fast(float x, const GroupScale& g) {
  FastCodes f = encode_candidate(x, g);
  if (__builtin_expect(f.off > kTie, 0)) f.c = encode(x, g.s, g.z);
  return f.c;
}

// Two elements behind one test: the rare path is entered half as often per element and still
// recomputes only the element that is near a tie.
__device__ __forceinline__ void encode_fast2(float x0, const GroupScale& g0, float x1, const GroupScale& g1,
                                             Codes& c0, Codes& c1) {
  FastCodes f0 = encode_candidate(x0, g0), f1 = encode_candidate(x1, g1);
  if (__builtin_expect(fmaxf(f0.off, f1.off) > kTie, 0)) {
    if (f0.off > kTie) f0.c = encode(x0, g0.s, g0.z);
    if (f1.off > kTie) f1.c = encode(x1, g1.s, g1.z);
  }
  c0 = f0.c;
  c1 = f1.c;
}

// Four 4-bit codes -> 16 bits of a plane word: acc += code * 16^k stays below 2^16, exact in binary32.
// The lower plane stores C_L + 8, so its accumulators start at 0x8888.
constexpr float kLowerBias = 34952.0f;
__device__ __forceinline__ void pack4(float& acc_u, float& acc_l, const Codes& c, int k) {
  const float w = (float)(1 << (4 * k));
  acc_u = __builtin_fmaf(c.u, w, acc_u);
  acc_l = __builtin_fmaf(c.l, w, acc_l);
}
__device__ __forceinline__ uint32_t packed_word(float lo16, float hi16) {
  return (uint32_t)lo16 | ((uint32_t)hi16 << 16);
}

// Key scale / zero are stored in the order the attention kernel's B operand wants them: position
// 32*s + 8*g + e of a group's 128 holds channel 32*g + 8*s + nibble(e).
__device__ __forceinline__ int key_meta_position(int ch) {
  const int g = ch >> 5, s = (ch >> 3) & 3, nib = ch & 7;
  return 32 * s + 8 * g + ((nib & 3) << 1) + (nib >> 2);
}

// Start of the cache block that holds token `tok` (unit-local) in the upper / lower array.
template <typename Args>
__device__ __forceinline__ auto upper_block(const Args& a, int unit, int tok) {
  return a.upper + (physical_group(a, unit, tok / kG) * (kG / kBlkTok) + (tok % kG) / kBlkTok) * kUpperBlk;
}
template <typename Args>
__device__ __forceinline__ auto lower_block(const Args& a, int unit, int tok) {
  return a.lower + (physical_group(a, unit, tok / kG) * (kG / kBlkTok) + (tok % kG) / kBlkTok) * kLowerBlk;
}
// Key scale / zero of channel ch of the group that starts at token tq0: k-step s = position / 32 of
// the group's operand order lives in the group's block s.
template <typename Args>
__device__ __forceinline__ void store_key_meta(const Args& a, int unit, int tq0, int ch, _Float16 s, _Float16 z) {
  const int pos = key_meta_position(ch);
  uint8_t* blk = upper_block(a, unit, tq0 + kBlkTok * (pos >> 5));
  reinterpret_cast<_Float16*>(blk + kOffKS)[pos & 31] = s;
  reinterpret_cast<_Float16*>(blk + kOffKZ)[pos & 31] = z;
}

// ------------------------------------------------------------------------------------------------
// Decode-time flush: four workgroups share one 128-token group of one unit so that a single flushed
// group already spreads over several compute units.  Workgroup q of the four handles
//   threads   0..127 : keys, channels [32q, 32q+32) of all 128 tokens, 16 channels per wave, so that a
//                      channel's minimum and maximum are found inside one wave
//   threads 128..255 : values, tokens [32q, 32q+32) (one value tile) of all 128 channels
// Each thread owns 4 channels of the eight tokens that share a value-plane word (32 codes).  The four waves
// meet only once, before the buffer move.  (With the keys' statistics going through LDS the two key waves
// waited at a workgroup barrier for the value waves' whole work and encoded after it: 9.3 us to the last
// store instead of 6.5 us.)
//
// Buffer move (Section 4.3.2), when the source is the buffer and one group is flushed: rows
// [128, n_buf) become rows [0, n_buf - 128) in the same launch.  Every buffer byte is read - as
// input of the quantization or as source of the move - only by the workgroup that overwrites it:
// workgroup q moves byte columns [64q, 64q+64) of the key rows (it alone quantizes them) and all
// columns of the value rows r with (r mod 128) / 32 = q (its value tile and the rows that land on
// it), and a thread keeps one row residue mod 128, so a row that is both destination and source is
// read and later written by the same thread.  The barrier before the move, behind every use of the
// quantization inputs, orders the reads of rows [0, 128) before the first store of the move.
__global__ __launch_bounds__(256) void flush_kernel(FlushArgs a) {
  const int grp = blockIdx.x >> 2, q = blockIdx.x & 3, unit = blockIdx.y;
  const int b = unit / a.n_kv_heads;
  const int tid = threadIdx.x;
  const int tq0 = a.n_quant[b] + grp * kG;     // destination token offset inside the unit
  const int64_t src0 = ((int64_t)unit * a.src_stride + (int64_t)grp * kG) * kD;

  // move: 64 bytes of one row per thread and round.  The first round's sources are fetched up front,
  // unconditionally (a thread with nothing to move reads a valid address and drops the data), so the
  // loads stay in flight under the quantization.
  const bool move = a.k_move != nullptr;
  const int n_keep = move ? a.n_buf[b] - kG : 0;
  const int mrow = tid < 128 ? tid : 32 * q + ((tid - 128) >> 2);
  _Float16* mcol = !move ? nullptr
                         : (tid < 128 ? a.k_move + 32 * q : a.v_move + 32 * (tid & 3)) + (int64_t)unit * a.src_stride * kD;
  const _Float16* mfirst = mrow < n_keep ? mcol + (int64_t)(mrow + kG) * kD : a.k_src + src0;
  auto load64 = [](const _Float16* p, uint4& x0, uint4& x1, uint4& x2, uint4& x3) {
    const uint4* w = reinterpret_cast<const uint4*>(p);
    x0 = w[0], x1 = w[1], x2 = w[2], x3 = w[3];
  };
  uint4 mv0, mv1, mv2, mv3;   // named registers: an array here is moved to LDS by the compiler
  load64(mfirst, mv0, mv1, mv2, mv3);

  if (tid < 128) {
    // ---- keys: min / max per channel over the 128 tokens of the group --------------------------
    const int c4 = tid & 3, oct = (tid & 63) >> 2, blk = oct >> 2, g = oct & 3;
    const int ch0 = 32 * q + 16 * (tid >> 6) + 4 * c4;
    half4 x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      x[j] = *reinterpret_cast<const half4*>(a.k_src + src0 + (int64_t)(32 * blk + tile_token(g, j)) * kD + ch0);
    float mn[4], mx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float lo = (float)x[0][i], hi = lo;
#pragma unroll
      for (int j = 1; j < 8; ++j) {
        lo = fminf(lo, (float)x[j][i]);
        hi = fmaxf(hi, (float)x[j][i]);
      }
#pragma unroll
      for (int sft = 4; sft < 64; sft <<= 1) {   // the sixteen octets of tokens, all in this wave
        lo = fminf(lo, __shfl_xor(lo, sft));
        hi = fmaxf(hi, __shfl_xor(hi, sft));
      }
      mn[i] = lo;
      mx[i] = hi;
    }
    GroupScale gs[4];
    _Float16 ksh[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ksh[i] = make_scale(mn[i], mx[i]);
      gs[i] = group_scale((float)ksh[i], mn[i]);
    }
    if (oct == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) store_key_meta(a, unit, tq0, ch0 + i, ksh[i], (_Float16)gs[i].z);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float wu = 0.0f, wl = kLowerBias;
#pragma unroll
      for (int i = 0; i < 4; ++i) pack4(wu, wl, encode_fast((float)x[j][i], gs[i]), i);
      const int tok = tq0 + 32 * blk + tile_token(g, j);
      const int off = kOffK + (tok % kBlkTok) * 64 + (ch0 >> 1);   // four channels = two bytes of the token's row
      *reinterpret_cast<uint16_t*>(upper_block(a, unit, tok) + off) = (uint16_t)(uint32_t)wu;
      *reinterpret_cast<uint16_t*>(lower_block(a, unit, tok) + off) = (uint16_t)(uint32_t)wl;
    }
  } else {
    // ---- values: min / max per token over its 128 channels --------------------------------------
    const int t = tid - 128, c4 = t & 31, g = t >> 5;
    half4 x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      x[j] = *reinterpret_cast<const half4*>(a.v_src + src0 + (int64_t)(32 * q + tile_token(g, j)) * kD + 4 * c4);
    half8 vsh, vzh;
    float vu[4][2], vl[4][2];   // per channel: nibbles 0..3 (even j) and 4..7 (odd j) of its plane word
#pragma unroll
    for (int i = 0; i < 4; ++i) vu[i][0] = vu[i][1] = 0.0f, vl[i][0] = vl[i][1] = kLowerBias;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float lo = (float)x[j][0], hi = lo;
#pragma unroll
      for (int i = 1; i < 4; ++i) {
        lo = fminf(lo, (float)x[j][i]);
        hi = fmaxf(hi, (float)x[j][i]);
      }
#pragma unroll
      for (int sft = 1; sft < 32; sft <<= 1) {   // the 32 lanes that hold the token's other channels
        lo = fminf(lo, __shfl_xor(lo, sft));
        hi = fmaxf(hi, __shfl_xor(hi, sft));
      }
      vsh[j] = make_scale(lo, hi);
      vzh[j] = (_Float16)lo;
      const GroupScale gs = group_scale((float)vsh[j], lo);
#pragma unroll
      for (int i = 0; i < 4; ++i) pack4(vu[i][j & 1], vl[i][j & 1], encode_fast((float)x[j][i], gs), j >> 1);
    }
    uint8_t* ub = upper_block(a, unit, tq0 + 32 * q);
    uint8_t* lb = lower_block(a, unit, tq0 + 32 * q);
    if (c4 == 0) {
      *reinterpret_cast<half8*>(ub + kOffVS + 16 * g) = vsh;
      *reinterpret_cast<half8*>(ub + kOffVZ + 16 * g) = vzh;
    }
    // channels 4*c4 .. 4*c4+3 = 8*m + 4*h + i with m = c4 >> 1, h = c4 & 1: four consecutive words
    const int w = kOffV + ((c4 & 1) * 64 + 16 * g + (c4 >> 1)) * 16;
    *reinterpret_cast<uint4*>(ub + w) = make_uint4(packed_word(vu[0][0], vu[0][1]), packed_word(vu[1][0], vu[1][1]),
                                                          packed_word(vu[2][0], vu[2][1]), packed_word(vu[3][0], vu[3][1]));
    *reinterpret_cast<uint4*>(lb + w) = make_uint4(packed_word(vl[0][0], vl[0][1]), packed_word(vl[1][0], vl[1][1]),
                                                          packed_word(vl[2][0], vl[2][1]), packed_word(vl[3][0], vl[3][1]));
  }
  if (move) __syncthreads();   // uniform over the workgroup: every quantization input has been read
  for (int r = mrow; r < n_keep; r += kG) {
    uint4* w = reinterpret_cast<uint4*>(mcol + (int64_t)r * kD);
    w[0] = mv0, w[1] = mv1, w[2] = mv2, w[3] = mv3;
    if (r + kG < n_keep) load64(mcol + (int64_t)(r + 2 * kG) * kD, mv0, mv1, mv2, mv3);
  }
}

// ------------------------------------------------------------------------------------------------
// Bulk quantization (prefill): one workgroup per 128-token group of one unit, every load issued
// before the first use, 8 channels x 8 tokens of K and of V per thread, whole rows per wave access
// (1 KB of source, 256 B of a plane per instruction).  Minima and maxima are taken on packed fp16
// pairs, which is exact.
//   keys:   thread (l16 = tid & 15, rg = tid >> 4) owns channels [8*l16, 8*l16+8) of tokens rg + 16*j;
//           channel statistics: in-thread over j, over the wave's four row groups, over the waves (LDS)
//   values: thread (l16, tg = tid >> 4) owns the same channels of the eight tokens that share the
//           plane words of value tile tg >> 2, lane group tg & 3; token statistics: in-thread over
//           the 8 channels, then over the 16 lanes of the row by rotation (min and -max side by side)
__device__ __forceinline__ half2 pmin(half2 a, half2 b) { return __builtin_elementwise_min(a, b); }
__device__ __forceinline__ half2 pmax(half2 a, half2 b) { return __builtin_elementwise_max(a, b); }
__device__ __forceinline__ half8 pmin(half8 a, half8 b) { return __builtin_elementwise_min(a, b); }
__device__ __forceinline__ half8 pmax(half8 a, half8 b) { return __builtin_elementwise_max(a, b); }

__device__ __forceinline__ half8 shfl_xor_h8(half8 v, int mask) {
  uint4 w = __builtin_bit_cast(uint4, v);
  w.x = __shfl_xor(w.x, mask);
  w.y = __shfl_xor(w.y, mask);
  w.z = __shfl_xor(w.z, mask);
  w.w = __shfl_xor(w.w, mask);
  return __builtin_bit_cast(half8, w);
}

template <int ROR>
__device__ __forceinline__ half2 row_rotate(half2 v) {   // lane i of each 16-lane row reads lane i + ROR (mod 16)
  const int w = __builtin_bit_cast(int, v);
  return __builtin_bit_cast(half2, __builtin_amdgcn_update_dpp(w, w, 0x120 + ROR, 0xF, 0xF, true));
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void quantize_group_kernel(FlushArgs a) {
  __shared__ uint4 part_lo[4][16], part_hi[4][16];   // per wave: 128 channel minima / maxima, fp16
  __shared__ float4 ksc[128];                        // per channel: S, Z, ~1/S, ~16/S
  const int grp = blockIdx.x, unit = blockIdx.y;
  const int b = unit / a.n_kv_heads;
  const int tid = threadIdx.x;
  const int tq0 = a.n_quant[b] + grp * kG;
  const int64_t src0 = ((int64_t)unit * a.src_stride + (int64_t)grp * kG) * kD;
  const int l16 = tid & 15, rg = tid >> 4;
  const int vtile = rg >> 2, vg = rg & 3;

  half8 xk[8], xv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) xk[j] = ld_half8(a.k_src + src0 + (int64_t)(rg + 16 * j) * kD + 8 * l16);
#pragma unroll
  for (int j = 0; j < 8; ++j)
    xv[j] = ld_half8(a.v_src + src0 + (int64_t)(32 * vtile + tile_token(vg, j)) * kD + 8 * l16);

  // ---- keys ------------------------------------------------------------------------------------
  {
    half8 lo = xk[0], hi = xk[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) {
      lo = pmin(lo, xk[j]);
      hi = pmax(hi, xk[j]);
    }
    lo = pmin(lo, shfl_xor_h8(lo, 16));
    hi = pmax(hi, shfl_xor_h8(hi, 16));
    lo = pmin(lo, shfl_xor_h8(lo, 32));
    hi = pmax(hi, shfl_xor_h8(hi, 32));
    if ((tid & 63) < 16) {
      part_lo[tid >> 6][l16] = __builtin_bit_cast(uint4, lo);
      part_hi[tid >> 6][l16] = __builtin_bit_cast(uint4, hi);
    }
  }
  __syncthreads();
  if (tid < 128) {
    const _Float16* pl = reinterpret_cast<const _Float16*>(&part_lo[0][0]);
    const _Float16* ph = reinterpret_cast<const _Float16*>(&part_hi[0][0]);
    float lo = (float)pl[tid], hi = (float)ph[tid];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      lo = fminf(lo, (float)pl[128 * w + tid]);
      hi = fmaxf(hi, (float)ph[128 * w + tid]);
    }
    const _Float16 sh = make_scale(lo, hi);
    const GroupScale gs = group_scale((float)sh, lo);
    ksc[tid] = make_float4(gs.s, gs.z, gs.r, gs.rl);
    store_key_meta(a, unit, tq0, tid, sh, (_Float16)lo);
  }
  __syncthreads();
  // two tokens at a time, the channel's (S, Z, 1/S, 16/S) read from LDS for each pair: this keeps
  // only eight packing accumulators live and releases the source registers as the tokens are done
#pragma unroll
  for (int j = 0; j < 8; j += 2) {
    float wu[2][2] = {{0.0f, 0.0f}, {0.0f, 0.0f}};   // [token of the pair][channels 0..3 / 4..7]
    float wl[2][2] = {{kLowerBias, kLowerBias}, {kLowerBias, kLowerBias}};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float4 m = ksc[8 * l16 + i];
      const GroupScale gs{m.x, m.y, m.z, m.w};
      Codes c0, c1;
      encode_fast2((float)xk[j][i], gs, (float)xk[j + 1][i], gs, c0, c1);
      pack4(wu[0][i >> 2], wl[0][i >> 2], c0, i & 3);
      pack4(wu[1][i >> 2], wl[1][i >> 2], c1, i & 3);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int tok = tq0 + rg + 16 * (j + t);
      const int off = kOffK + (tok % kBlkTok) * 64 + 4 * l16;
      *reinterpret_cast<uint32_t*>(upper_block(a, unit, tok) + off) = packed_word(wu[t][0], wu[t][1]);
      *reinterpret_cast<uint32_t*>(lower_block(a, unit, tok) + off) = packed_word(wl[t][0], wl[t][1]);
    }
  }
  // ---- values ------------------------------------------------------------------------------------
  {
    half8 vsh, vzh;
    float vu[8][2], vl[8][2];   // per channel: nibbles 0..3 (even j) and 4..7 (odd j) of its plane word
#pragma unroll
    for (int i = 0; i < 8; ++i) vu[i][0] = vu[i][1] = 0.0f, vl[i][0] = vl[i][1] = kLowerBias;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const half8 x = xv[j];
      const half2 x01 = x.s01, x23 = x.s23, x45 = x.s45, x67 = x.s67;
      const half2 mn2 = pmin(pmin(x01, x23), pmin(x45, x67));
      const half2 mx2 = pmax(pmax(x01, x23), pmax(x45, x67));
      half2 p = pmin(half2{mn2.x, -mx2.x}, half2{mn2.y, -mx2.y});   // (min, -max) of the 8 channels
      p = pmin(p, row_rotate<1>(p));
      p = pmin(p, row_rotate<2>(p));
      p = pmin(p, row_rotate<4>(p));
      p = pmin(p, row_rotate<8>(p));
      const float lo = (float)p.x, hi = -(float)p.y;
      vsh[j] = make_scale(lo, hi);
      vzh[j] = p.x;
      const GroupScale gs = group_scale((float)vsh[j], lo);
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        Codes c0, c1;
        encode_fast2((float)x[i], gs, (float)x[i + 1], gs, c0, c1);
        pack4(vu[i][j & 1], vl[i][j & 1], c0, j >> 1);
        pack4(vu[i + 1][j & 1], vl[i + 1][j & 1], c1, j >> 1);
      }
    }
    uint8_t* ub = upper_block(a, unit, tq0 + 32 * vtile);
    uint8_t* lb = lower_block(a, unit, tq0 + 32 * vtile);
    if (l16 == 0) {
      *reinterpret_cast<half8*>(ub + kOffVS + 16 * vg) = vsh;
      *reinterpret_cast<half8*>(ub + kOffVZ + 16 * vg) = vzh;
    }
    // channel 8*l16 + 4*h + i lives in word (h*64 + 16*vg + l16)*4 + i of the tile
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int w = kOffV + (h * 64 + 16 * vg + l16) * 16;
      *reinterpret_cast<uint4*>(ub + w) =
          make_uint4(packed_word(vu[4 * h][0], vu[4 * h][1]), packed_word(vu[4 * h + 1][0], vu[4 * h + 1][1]),
                     packed_word(vu[4 * h + 2][0], vu[4 * h + 2][1]), packed_word(vu[4 * h + 3][0], vu[4 * h + 3][1]));
      *reinterpret_cast<uint4*>(lb + w) =
          make_uint4(packed_word(vl[4 * h][0], vl[4 * h][1]), packed_word(vl[4 * h + 1][0], vl[4 * h + 1][1]),
                     packed_word(vl[4 * h + 2][0], vl[4 * h + 2][1]), packed_word(vl[4 * h + 3][0], vl[4 * h + 3][1]));
    }
  }
}

// Buffer move (Section 4.3.2): rows [n_tokens, n_buf) become rows [0, n_buf - n_tokens).  Source and
// destination may overlap.  Thread (rl = tid >> 4, c = tid & 15) of the 1024 moves rows rl, rl+64, ...
// of its own 16-byte column; n_tokens is a multiple of 64, so a row is only ever overwritten by the
// thread that read it as a source, and no cross-thread ordering is needed.  Up to four rows per
// thread are read before the first one is written, so a typical move is one memory round trip.
__global__ __launch_bounds__(1024) void shift_kernel(ShiftArgs a) {
  const int unit = blockIdx.x;
  const int b = unit / a.n_kv_heads;
  _Float16* buf = (blockIdx.y == 0 ? a.k_buf : a.v_buf) + (int64_t)unit * a.buf_cap * kD;
  const int n_keep = a.n_buf[b] - a.n_tokens;
  const int c = threadIdx.x & 15, rl = threadIdx.x >> 4;
  for (int base = rl; base < n_keep; base += 256) {
    uint4 x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int r = min(base + 64 * k, n_keep - 1);
      x[k] = *reinterpret_cast<const uint4*>(buf + (int64_t)(r + a.n_tokens) * kD + 8 * c);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (base + 64 * k < n_keep) *reinterpret_cast<uint4*>(buf + (int64_t)(base + 64 * k) * kD + 8 * c) = x[k];
  }
}

// Append: one 16-byte chunk per thread, [B][n_new][Hkv][head_dim] -> buffer rows n_buf[b] .. of every unit.
__global__ __launch_bounds__(256) void append_kernel(AppendArgs a) {
  const int b = blockIdx.y;
  const int idx = blockIdx.x * 256 + threadIdx.x;           // (token, kv-head, 16-byte chunk)
  const int d = a.head_dim, cpr = d / 8;                    // chunks per row
  const int per_tok = a.n_kv_heads * cpr;
  if (idx >= a.n_new * per_tok) return;
  const int tok = idx / per_tok, h = (idx % per_tok) / cpr, c = idx % cpr;
  const int64_t src = (((int64_t)b * a.n_new + tok) * a.n_kv_heads + h) * d + 8 * c;
  const int64_t dst = (((int64_t)b * a.n_kv_heads + h) * a.buf_cap + a.n_buf[b] + tok) * d + 8 * c;
  *reinterpret_cast<uint4*>(a.k_buf + dst) = *reinterpret_cast<const uint4*>(a.k_new + src);
  *reinterpret_cast<uint4*>(a.v_buf + dst) = *reinterpret_cast<const uint4*>(a.v_new + src);
}

// Expand the blocked arrays of one unit into one code per byte, plain [token][channel] order.
__global__ __launch_bounds__(256) void export_kernel(ExportArgs a) {
  const int idx = blockIdx.x * 256 + threadIdx.x;      // one 32-bit word of key codes and one of value codes
  if (idx >= a.n_tokens * kRowDw) return;
  const int blk = idx >> 9, w = idx & 511;             // 512 words of either kind per 32-token block
  const uint8_t* ub = upper_block(a, a.unit, kBlkTok * blk);
  const uint8_t* lb = lower_block(a, a.unit, kBlkTok * blk);
  {  // keys: word w of the block = row (w >> 4), channels 8*(w & 15) ..
    const int tok = 32 * blk + (w >> 4), c8 = w & 15;
    const uint32_t wu = *reinterpret_cast<const uint32_t*>(ub + kOffK + 4 * w);
    const uint32_t wl = *reinterpret_cast<const uint32_t*>(lb + kOffK + 4 * w);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (a.k_u) a.k_u[tok * kD + 8 * c8 + i] = (uint8_t)((wu >> (4 * i)) & 15u);
      if (a.k_l) a.k_l[tok * kD + 8 * c8 + i] = (int8_t)((int)((wl >> (4 * i)) & 15u) - 8);
    }
  }
  {  // values: word w = (h*64 + 16*g + m)*4 + i of the tile
    const int h = w >> 8, g = (w >> 6) & 3, m = (w >> 2) & 15, i = w & 3;
    const int ch = 8 * m + 4 * h + i;
    const uint32_t wu = *reinterpret_cast<const uint32_t*>(ub + kOffV + 4 * w);
    const uint32_t wl = *reinterpret_cast<const uint32_t*>(lb + kOffV + 4 * w);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok = 32 * blk + tile_token(g, j);
      const int nib = 4 * tile_nibble(j);
      if (a.v_u) a.v_u[tok * kD + ch] = (uint8_t)((wu >> nib) & 15u);
      if (a.v_l) a.v_l[tok * kD + ch] = (int8_t)((int)((wl >> nib) & 15u) - 8);
    }
  }
  if (w < 32) {  // key metadata: position 32*s + 8*g + e of a group (s = block mod 4) -> channel 32*g + 8*s + nibble(e)
    const int grp = blk >> 2, s = blk & 3;
    const int ch = 32 * (w >> 3) + 8 * s + tile_nibble(w & 7);
    if (a.k_s) a.k_s[grp * kD + ch] = reinterpret_cast<const _Float16*>(ub + kOffKS)[w];
    if (a.k_z) a.k_z[grp * kD + ch] = reinterpret_cast<const _Float16*>(ub + kOffKZ)[w];
    // value metadata: position 8*g + j of the block -> token order
    const int tok = 32 * blk + tile_token(w >> 3, w & 7);
    if (a.v_s) a.v_s[tok] = reinterpret_cast<const _Float16*>(ub + kOffVS)[w];
    if (a.v_z) a.v_z[tok] = reinterpret_cast<const _Float16*>(ub + kOffVZ)[w];
  }
}


// ------------------------------------------------------------------------------------------------
// Other shapes than head_dim = group = 128: the plain layout (superblocks of 128 tokens, see
// quantspec.h).  One workgroup per (unit, G-token key group); the same encoding, written for clarity
// rather than speed: codes are staged one per byte in LDS and packed from there.
//   keys:   thread (c = tid % D, slice = tid / D) walks the group's tokens slice, slice + 256/D, ...
//           of channel c twice - statistics, then codes with the group's (S, Z)
//   values: one thread per (token, value group of G channels): D of them for G tokens
// ------------------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(256) void quantize_plain_kernel(FlushArgs a) {
  constexpr int C8 = D / 8;       // 16-byte pieces (eight channels) of a token row
  constexpr int RPP = 256 / C8;   // token rows the 256 threads cover at a time (at most 32, so never more than G)
  constexpr int VG = D / G;       // value groups per token
  constexpr int LPG = G / 8;      // threads that share a value group: consecutive lanes of one wave
  __shared__ uint8_t cb[G][D];    // staged codes, one element per byte: C_U in the low nibble, C_L + 8 in the high one
  __shared__ float red[2][RPP][D];
  __shared__ float kmeta[2][D];   // key scale and zero of the group, per channel
  const ShapeLayout lay{D, G};
  const int grp = blockIdx.x, unit = blockIdx.y;
  const int b = unit / a.n_kv_heads;
  const int tid = threadIdx.x;
  const int c8 = tid % C8, r0 = tid / C8;          // this thread's piece of the rows r0, r0 + RPP, ...
  const int tq0 = a.n_quant[b] + grp * G;          // destination token offset inside the unit (multiple of G)
  const int64_t src0 = ((int64_t)unit * a.src_stride + (int64_t)grp * G) * D + 8 * c8;
  const int sb_tok = tq0 % kSuper;                 // first token of the group inside its 128-token row of the layout
  uint8_t* ub = a.upper + physical_group(a, unit, tq0 / kSuper) * lay.upper_bytes();
  uint8_t* lb = a.lower + physical_group(a, unit, tq0 / kSuper) * lay.lower_bytes();
  using half8v = _Float16 __attribute__((ext_vector_type(8)));
  auto stage = [&](int t, const Codes (&cd)[8]) {   // eight codes of row t -> eight staging bytes
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i >> 2] |= ((uint32_t)cd[i].u | ((uint32_t)(cd[i].l + 8.0f) << 4)) << (8 * (i & 3));
    *reinterpret_cast<uint2*>(&cb[t][8 * c8]) = make_uint2(w[0], w[1]);
  };

  // staged codes -> the words of the group's 32-token blocks, in the order the attention kernel's lanes load
  // them (see ShapeLayout): consecutive threads write consecutive words
  auto pack = [&](bool values) {
    constexpr int WPB = 4 * D;   // words per block and kind
    for (int w = tid; w < (G / 32) * WPB; w += 256) {
      const int bl = w / WPB, r = w % WPB;
      uint32_t wu = 0, wl = 0;
      if (!values) {
        constexpr int KS = D / 32;   // word r -> (t, lane, s): the inverse of ShapeLayout::k_word
        const int lane = (r / 4) % 64;
        const int s = KS == 2 ? r % 2 : 4 * ((r / 256) % (KS / 4)) + r % 4, t = KS == 2 ? (r / 2) % 2 : r / (64 * KS);
        const int tok = 32 * bl + 16 * t + (lane & 15), c0 = 32 * s + 8 * (lane >> 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) wu |= (uint32_t)(cb[tok][c0 + i] & 15) << (4 * tile_nibble(i)), wl |= (uint32_t)(cb[tok][c0 + i] >> 4) << (4 * tile_nibble(i));
      } else {
        const int lane = (r / 4) % 64, n = 4 * (r / 256) + r % 4;
        const int c = 16 * n + (lane & 15), tok0 = 32 * bl + 4 * (lane >> 4);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t code = cb[tok0 + 16 * (j >> 2) + (j & 3)][c];
          wu |= (code & 15u) << (4 * tile_nibble(j)), wl |= (code >> 4) << (4 * tile_nibble(j));
        }
      }
      const int off = (values ? lay.off_v(sb_tok / 32 + bl) : lay.off_k(sb_tok / 32 + bl)) + 4 * r;
      *reinterpret_cast<uint32_t*>(ub + off) = wu;
      *reinterpret_cast<uint32_t*>(lb + off) = wl;
    }
  };

  // ---- keys: per channel over the G tokens ----
  {
    float lo[8], hi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) lo[i] = __builtin_inff(), hi[i] = -__builtin_inff();
    for (int t = r0; t < G; t += RPP) {
      const half8v x = *reinterpret_cast<const half8v*>(a.k_src + src0 + (int64_t)t * D);
#pragma unroll
      for (int i = 0; i < 8; ++i) lo[i] = fminf(lo[i], (float)x[i]), hi[i] = fmaxf(hi[i], (float)x[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[0][r0][8 * c8 + i] = lo[i], red[1][r0][8 * c8 + i] = hi[i];
    __syncthreads();
    if (tid < D) {
      float l = red[0][0][tid], h = red[1][0][tid];
#pragma unroll
      for (int k = 1; k < RPP; ++k) l = fminf(l, red[0][k][tid]), h = fmaxf(h, red[1][k][tid]);
      const _Float16 sh = make_scale(l, h);
      kmeta[0][tid] = (float)sh, kmeta[1][tid] = l;
      reinterpret_cast<_Float16*>(ub + lay.off_ks())[(sb_tok / G) * D + tid] = sh;
      reinterpret_cast<_Float16*>(ub + lay.off_kz())[(sb_tok / G) * D + tid] = (_Float16)l;
    }
    __syncthreads();
    GroupScale gs[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) gs[i] = group_scale(kmeta[0][8 * c8 + i], kmeta[1][8 * c8 + i]);
    for (int t = r0; t < G; t += RPP) {
      const half8v x = *reinterpret_cast<const half8v*>(a.k_src + src0 + (int64_t)t * D);
      Codes cd[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) cd[i] = encode_fast((float)x[i], gs[i]);
      stage(t, cd);
    }
  }
  __syncthreads();
  pack(false);
  __syncthreads();
  // ---- values: per token over each group of G channels, LPG threads to a group ----
  for (int t = r0; t < G; t += RPP) {   // the same number of rounds for every thread
    const half8v x = *reinterpret_cast<const half8v*>(a.v_src + src0 + (int64_t)t * D);
    float lo = (float)x[0], hi = lo;
#pragma unroll
    for (int i = 1; i < 8; ++i) lo = fminf(lo, (float)x[i]), hi = fmaxf(hi, (float)x[i]);
#pragma unroll
    for (int m = 1; m < LPG; m <<= 1) lo = fminf(lo, __shfl_xor(lo, m)), hi = fmaxf(hi, __shfl_xor(hi, m));
    const _Float16 sh = make_scale(lo, hi);
    const GroupScale gs = group_scale((float)sh, lo);
    if (c8 % LPG == 0) {
      reinterpret_cast<_Float16*>(ub + lay.off_vs())[(sb_tok + t) * VG + c8 / LPG] = sh;
      reinterpret_cast<_Float16*>(ub + lay.off_vz())[(sb_tok + t) * VG + c8 / LPG] = (_Float16)lo;
    }
    Codes cd[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) cd[i] = encode_fast((float)x[i], gs);
    stage(t, cd);
  }
  __syncthreads();
  pack(true);
}

// Buffer move for any head_dim: rows [n_tokens, n_buf) become rows [0, n_buf - n_tokens).  Thread
// (rl = tid / (D/8), c) moves rows rl, rl + 32, ... of its 16-byte column, four at a time; n_tokens is a
// multiple of 32, so a row is only overwritten by the thread that read it as a source before.
template <int D>
__global__ __launch_bounds__(4 * D) void shift_plain_kernel(ShiftArgs a) {
  constexpr int COLS = D / 8;
  const int unit = blockIdx.x;
  const int b = unit / a.n_kv_heads;
  _Float16* buf = (blockIdx.y == 0 ? a.k_buf : a.v_buf) + (int64_t)unit * a.buf_cap * D;
  const int n_keep = a.n_buf[b] - a.n_tokens;
  const int c = threadIdx.x % COLS, rl = threadIdx.x / COLS;
  for (int base = rl; base < n_keep; base += 128) {
    uint4 x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int r = min(base + 32 * k, n_keep - 1);
      x[k] = *reinterpret_cast<const uint4*>(buf + (int64_t)(r + a.n_tokens) * D + 8 * c);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (base + 32 * k < n_keep) *reinterpret_cast<uint4*>(buf + (int64_t)(base + 32 * k) * D + 8 * c) = x[k];
  }
}

// Plain layout -> one code per byte and metadata in [token][channel] order (see export_kernel).
template <int D, int G>
__global__ __launch_bounds__(256) void export_plain_kernel(ExportArgs a) {
  constexpr int VG = D / G;
  const ShapeLayout lay{D, G};
  const int idx = blockIdx.x * 256 + threadIdx.x;      // eight channels of one token
  if (idx >= a.n_tokens * (D / 8)) return;
  const int tok = idx / (D / 8), c0 = 8 * (idx % (D / 8));
  const uint8_t* ub = a.upper + physical_group(a, a.unit, tok / kSuper) * lay.upper_bytes();
  const uint8_t* lb = a.lower + physical_group(a, a.unit, tok / kSuper) * lay.lower_bytes();
  const int p = (tok % kSuper) / 32, tl = tok % 32, t = tl / 16;
  {   // keys: the eight channels are the eight nibbles of one word, channel i in nibble tile_nibble(i)
    const int off = lay.off_k(p) + 4 * lay.k_word(t, 16 * ((c0 / 8) % 4) + tl % 16, c0 / 32);
    const uint32_t wu = *reinterpret_cast<const uint32_t*>(ub + off);
    const uint32_t wl = *reinterpret_cast<const uint32_t*>(lb + off);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (a.k_u) a.k_u[(int64_t)tok * D + c0 + i] = (uint8_t)((wu >> (4 * tile_nibble(i))) & 15u);
      if (a.k_l) a.k_l[(int64_t)tok * D + c0 + i] = (int8_t)((int)((wl >> (4 * tile_nibble(i))) & 15u) - 8);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {   // values: one word per channel, the token picks the nibble
    const int c = c0 + i, j = tile_nibble(4 * t + tl % 4);
    const int off = lay.off_v(p) + 4 * lay.v_word(c / 16, 16 * ((tl % 16) / 4) + c % 16);
    const uint32_t wu = *reinterpret_cast<const uint32_t*>(ub + off);
    const uint32_t wl = *reinterpret_cast<const uint32_t*>(lb + off);
    if (a.v_u) a.v_u[(int64_t)tok * D + c] = (uint8_t)((wu >> (4 * j)) & 15u);
    if (a.v_l) a.v_l[(int64_t)tok * D + c] = (int8_t)((int)((wl >> (4 * j)) & 15u) - 8);
  }
  if (tok % G == 0) {   // key metadata of the token's group: this thread's eight channels
    const _Float16* ks = reinterpret_cast<const _Float16*>(ub + lay.off_ks()) + ((tok % kSuper) / G) * D;
    const _Float16* kz = reinterpret_cast<const _Float16*>(ub + lay.off_kz()) + ((tok % kSuper) / G) * D;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (a.k_s) a.k_s[(int64_t)(tok / G) * D + c0 + i] = ks[c0 + i];
      if (a.k_z) a.k_z[(int64_t)(tok / G) * D + c0 + i] = kz[c0 + i];
    }
  }
  if (c0 % G == 0) {    // value metadata of the group that starts at this thread's first channel
    const int vg = c0 / G;
    if (a.v_s) a.v_s[(int64_t)tok * VG + vg] = reinterpret_cast<const _Float16*>(ub + lay.off_vs())[(tok % kSuper) * VG + vg];
    if (a.v_z) a.v_z[(int64_t)tok * VG + vg] = reinterpret_cast<const _Float16*>(ub + lay.off_vz())[(tok % kSuper) * VG + vg];
  }
}

// ------------------------------------------------------------------------------------------------
// 4-bit weights of the draft model's linear layers (see quantspec.h): the quantizer above, one group per
// output row and 128 input channels.  One workgroup per block of 16 rows x 128 channels; thread (r, c)
// takes channels 8c .. 8c+7 of row r, which are exactly the eight codes of one word of the layout.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void w4_quantize_kernel(W4Args a) {
  const int groups = a.n_in / 128;
  const int T = blockIdx.x / groups, g = blockIdx.x % groups;
  const int r = threadIdx.x >> 4, c = threadIdx.x & 15;
  const half8 x = ld_half8(a.w + (int64_t)(16 * T + r) * a.n_in + 128 * g + 8 * c);
  float lo = (float)x[0], hi = lo;
#pragma unroll
  for (int i = 1; i < 8; ++i) lo = fminf(lo, (float)x[i]), hi = fmaxf(hi, (float)x[i]);
#pragma unroll
  for (int m = 1; m < 16; m <<= 1) lo = fminf(lo, __shfl_xor(lo, m)), hi = fmaxf(hi, __shfl_xor(hi, m));
  const _Float16 sh = make_scale(lo, hi);
  const GroupScale gs = group_scale((float)sh, lo);
  uint32_t word = 0u;
#pragma unroll
  for (int i = 0; i < 8; ++i) word |= (uint32_t)encode_fast((float)x[i], gs).u << (4 * tile_nibble(i));
  uint8_t* blk = a.packed + (int64_t)blockIdx.x * kW4Codes;
  const int lane = 16 * (c & 3) + r, s = c >> 2;
  reinterpret_cast<uint32_t*>(blk)[lane * 4 + s] = word;
  if (c == 0) {   // rows 4a .. 4a+3 keep S (8 bytes) and Z (8 bytes) side by side
    _Float16* meta = reinterpret_cast<_Float16*>(a.packed + w4_meta_base(a.n_out, a.n_in) + (int64_t)blockIdx.x * kW4Meta);
    meta[8 * (r >> 2) + (r & 3)] = sh;
    meta[8 * (r >> 2) + 4 + (r & 3)] = (_Float16)lo;
  }
}

// Packed weights -> one code per byte [n_out][n_in], scales and zeros [n_out][n_in / 128].
__global__ __launch_bounds__(256) void w4_export_kernel(W4Args a) {
  const int groups = a.n_in / 128;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;      // eight channels of one row
  if (idx >= (int64_t)a.n_out * (a.n_in / 8)) return;
  const int n = (int)(idx / (a.n_in / 8)), c8 = (int)(idx % (a.n_in / 8));
  const int g = c8 / 16, c = c8 % 16, r = n % 16;
  const int64_t block = (int64_t)(n / 16) * groups + g;
  const uint8_t* blk = a.packed + block * kW4Codes;
  const _Float16* meta = reinterpret_cast<const _Float16*>(a.packed + w4_meta_base(a.n_out, a.n_in) + block * kW4Meta);
  const uint32_t word = reinterpret_cast<const uint32_t*>(blk)[(16 * (c & 3) + r) * 4 + (c >> 2)];
  if (a.codes != nullptr) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a.codes[(int64_t)n * a.n_in + 8 * c8 + i] = (uint8_t)((word >> (4 * tile_nibble(i))) & 15u);
  }
  if (c == 0) {
    if (a.scale != nullptr) a.scale[(int64_t)n * groups + g] = meta[8 * (r >> 2) + (r & 3)];
    if (a.zero != nullptr) a.zero[(int64_t)n * groups + g] = meta[8 * (r >> 2) + 4 + (r & 3)];
  }
}

// Calls f with the compile-time shape that matches (d, g); false if the shape is not built.
template <typename F>
bool with_shape(int d, int g, F&& f) {
#define QS_SHAPE(DD, GG)                                                          \
  if (d == DD && g == GG) {                                                       \
    f(std::integral_constant<int, DD>{}, std::integral_constant<int, GG>{});     \
    return true;                                                                  \
  }
  QS_SHAPE(64, 32) QS_SHAPE(64, 64) QS_SHAPE(128, 32) QS_SHAPE(128, 64) QS_SHAPE(256, 32) QS_SHAPE(256, 64) QS_SHAPE(256, 128)
#undef QS_SHAPE
  return false;
}

}  // namespace

bool flush_moves_buffer(int head_dim, int group, int n_groups, int units) {
  return head_dim == kD && group == kG && n_groups == 1 && units < kBulkGroups;
}

hipError_t launch_flush(const FlushArgs& a, int batch, hipStream_t s) {
  if (a.n_groups <= 0) return hipSuccess;
  const int units = batch * a.n_kv_heads;
  if (a.head_dim != kD || a.group != kG) {   // n_groups counts groups of a.group tokens here
    hipError_t rc = hipErrorInvalidValue;
    with_shape(a.head_dim, a.group, [&](auto DD, auto GG) {
      rc = launch(quantize_plain_kernel<decltype(DD)::value, decltype(GG)::value>, dim3(a.n_groups, units), dim3(256), s, a);
    });
    return rc;
  }
  if ((int64_t)a.n_groups * units >= kBulkGroups)
    return launch(quantize_group_kernel, dim3(a.n_groups, units), dim3(256), s, a);
  return launch(flush_kernel, dim3(4 * a.n_groups, units), dim3(256), s, a);
}

hipError_t launch_shift(const ShiftArgs& a, int batch, hipStream_t s) {
  dim3 grid(batch * a.n_kv_heads, 2);
  if (a.head_dim == 64) return launch(shift_plain_kernel<64>, grid, dim3(256), s, a);
  if (a.head_dim == 256) return launch(shift_plain_kernel<256>, grid, dim3(1024), s, a);
  if (a.n_tokens % 64 != 0) return launch(shift_plain_kernel<128>, grid, dim3(512), s, a);   // groups of 32 tokens
  return launch(shift_kernel, grid, dim3(1024), s, a);
}

hipError_t launch_append(const AppendArgs& a, int batch, hipStream_t s) {
  const int chunks = a.n_new * a.n_kv_heads * (a.head_dim / 8);
  return launch(append_kernel, dim3((chunks + 255) / 256, batch), dim3(256), s, a);
}

hipError_t launch_export(const ExportArgs& a, hipStream_t s) {
  if (a.n_tokens <= 0) return hipSuccess;
  if (a.head_dim != kD || a.group != kG) {
    hipError_t rc = hipErrorInvalidValue;
    with_shape(a.head_dim, a.group, [&](auto DD, auto GG) {
      constexpr int D = decltype(DD)::value;
      rc = launch(export_plain_kernel<D, decltype(GG)::value>, dim3((a.n_tokens * (D / 8) + 255) / 256), dim3(256), s, a);
    });
    return rc;
  }
  const int words = a.n_tokens * kRowDw;
  return launch(export_kernel, dim3((words + 255) / 256), dim3(256), s, a);
}

hipError_t launch_w4_quantize(const W4Args& a, hipStream_t s) {
  return launch(w4_quantize_kernel, dim3((a.n_out / 16) * (a.n_in / 128)), dim3(256), s, a);
}

hipError_t launch_w4_export(const W4Args& a, hipStream_t s) {
  const int64_t items = (int64_t)a.n_out * (a.n_in / 8);
  return launch(w4_export_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), s, a);
}

}  // namespace qs
