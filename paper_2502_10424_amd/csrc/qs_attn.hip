// Split-K decode attention over the hierarchical 4-bit KV cache (gfx950, wave64, MFMA).
//
// Draft pass (paper Section 4.2 / Algorithm 1 DRAFT): keys and values are decoded from the upper
// plane only, x = C_U*S + Z.  Verify pass (TARGET): both planes, x = (16*C_U + C_L)*(S/16) + Z.
// Both also attend the full-precision buffer (Section 4.3.2), which is one more chunk of the
// split-K scheme (Appendix E), and every chunk's (max, sum, output) partial is merged afterwards.
//
// Design
//  * One wave walks 128-token groups of one (sequence, kv-head) unit for all query rows that share
//    that kv-head (grouped-query heads x query tokens), so the planes are read once, and writes one
//    partial.  Either every wave is a workgroup with a fixed contiguous range (attn_kernel; one wave per
//    SIMD by default), or the eight waves of a compute unit form one workgroup and draw their groups from a
//    queue in LDS (attn_kernel_cu: the two waves of a SIMD do not advance at the same pace).
//    Every byte of the planes is loaded exactly once, by exactly one lane, with 128-bit loads that a
//    wave issues as contiguous 1 KB requests, directly into the registers that feed the matrix cores;
//    the cache is laid out in 32-token blocks so that these requests walk one array (draft) or two
//    (verify) front to back.  LDS is only used to transpose the fp16 value tiles of the buffer chunk.
//  * The contraction runs on the matrix cores (v_mfma_f32_16x16x32_f16): codes are the A operand,
//    queries / probabilities the B operand.  Scales never touch individual codes:
//        q . K_hat[t] = sum_d (q_d S_d) c[t,d] + q . Z          (per 128-token group)
//        o            = sum_t (p_t S_t) c[t,:] + sum_t p_t Z_t  (per token)
//  * A 4-bit code masked in place inside its 32-bit word is already an fp16 subnormal
//    (c * 2^-24 for bits 0-3 of a half, c * 2^-20 for bits 4-7); the matrix cores take subnormal
//    inputs exactly, so "dequantization" is one AND per two codes and the powers of two are folded
//    into the other operand and the final scale.
//  * q_d S_d is split exactly into an fp16 high part and an fp16 remainder that occupy two columns
//    of the same 16-column MFMA tile (8 query rows + 8 remainders), so key metadata costs no accuracy.
//  * The MFMA output layout of Q K^T (lane = query column, 4 consecutive tokens) is, after packing to
//    fp16, directly the B operand layout of P V; the value planes are stored by the flush kernel in
//    exactly the token order this produces, so probabilities never cross lanes.
#include <type_traits>

#include "qs_internal.h"

namespace qs {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ half8 as_half8(u32x4 v) { return __builtin_bit_cast(half8, v); }
__device__ __forceinline__ u32x4 as_u32x4(half8 v) { return __builtin_bit_cast(u32x4, v); }
__device__ __forceinline__ half2v as_half2(uint32_t v) { return __builtin_bit_cast(half2v, v); }
__device__ __forceinline__ uint32_t as_u32(half2v v) { return __builtin_bit_cast(uint32_t, v); }

__device__ __forceinline__ u32x4 ldg128(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
// The same for data that is read once per launch and is far larger than the caches (the planes and
// their metadata): a non-temporal load leaves the L2 and the memory-side cache to the data that is
// reused (queries, buffer, partials).  Measured at 128k context: draft call 103 -> 95 us, verify
// call 196 -> 174 us.  (The fp16 buffer, whose 64-byte pieces share cache lines between
// instructions, and the prefill quantizer, which is bound by arithmetic, gain nothing from it.)
__device__ __forceinline__ u32x4 ldg128_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
// One 32-token block of a plane as a buffer resource: the block's address is uniform over the wave and
// sits in the descriptor, a lane adds a 32-bit offset that never changes, so a load needs no address
// arithmetic, and the hardware returns zero instead of reading past the block.  Non-temporal as above
// (cache-policy bit 1); a loads-only probe streams another 5 % faster this way than through 64-bit
// global addresses.
constexpr int kBufferWord3 = 0x00020000;   // raw 32-bit elements (gfx9 family)
constexpr int kAuxStream = 2;              // nt
__device__ __forceinline__ __amdgpu_buffer_rsrc_t block_resource(const uint8_t* block, int bytes) {
  // the address is the same in every lane; saying so keeps the descriptor in scalar registers
  const uint64_t p = reinterpret_cast<uint64_t>(block);
  const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<uint8_t*>((hi << 32) | lo), 0, bytes, kBufferWord3);
}
__device__ __forceinline__ u32x4 ldb128_stream(__amdgpu_buffer_rsrc_t r, int off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, kAuxStream);
}
__device__ __forceinline__ u32x4 ldb128(__amdgpu_buffer_rsrc_t r, int off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
}
__device__ __forceinline__ uint32_t ldb16_stream(__amdgpu_buffer_rsrc_t r, int off) {
  return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, off, 0, kAuxStream);
}

// Eight 4-bit codes of one word -> eight fp16 subnormals.  Operand element j comes from nibble
// (j&1)*4 + (j>>1); elements 2,3,6,7 carry an extra factor 16 (bits 4-7 of their half).
__device__ __forceinline__ half8 unpack4(uint32_t x) {
  const uint32_t y = x >> 8;
  u32x4 r;
  r[0] = x & 0x000F000Fu;
  r[1] = x & 0x00F000F0u;
  r[2] = y & 0x000F000Fu;
  r[3] = y & 0x00F000F0u;
  return as_half8(r);
}

// Upper and lower nibbles -> eight 8-bit codes 16*C_U + (C_L + 8) as fp16 subnormals (x 2^-24),
// same element order as unpack4.
__device__ __forceinline__ half8 unpack8(uint32_t u, uint32_t l) {
  uint32_t even = ((u << 4) & 0xF0F0F0F0u) | (l & 0x0F0F0F0Fu);   // nibbles 0,2,4,6 -> bytes 0..3
  uint32_t odd = (u & 0xF0F0F0F0u) | ((l >> 4) & 0x0F0F0F0Fu);    // nibbles 1,3,5,7 -> bytes 0..3
  // keep the two merged words as they are: folding the masks below into their construction costs
  // four more instructions per call than using them (8 instead of 12 for eight codes)
  asm volatile("" : "+v"(even), "+v"(odd));
  u32x4 r;
  r[0] = even & 0x00FF00FFu;                                  // nibbles 0, 4
  r[1] = odd & 0x00FF00FFu;                                   // nibbles 1, 5
  r[2] = __builtin_amdgcn_perm(0u, even, 0x0c030c01u);        // nibbles 2, 6
  r[3] = __builtin_amdgcn_perm(0u, odd, 0x0c030c01u);         // nibbles 3, 7
  return as_half8(r);
}

// Reorder eight consecutive channels so that element j holds channel (j&1)*4 + (j>>1), i.e. the
// channel whose code unpack4/unpack8 deliver at element j.
__device__ __forceinline__ half8 to_operand_order(half8 c) {
  half8 r;
  r[0] = c[0]; r[1] = c[4]; r[2] = c[1]; r[3] = c[5];
  r[4] = c[2]; r[5] = c[6]; r[6] = c[3]; r[7] = c[7];
  return r;
}

__device__ __forceinline__ float group_max(float x) {     // over the four 16-lane groups of the wave
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float group_sum(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}
__device__ __forceinline__ float pow2(int e) { return __builtin_bit_cast(float, (uint32_t)(127 + e) << 23); }   // -126 <= e <= 127
__device__ __forceinline__ int exponent_of(float x) { return (int)((__builtin_bit_cast(uint32_t, x) >> 23) & 255u) - 127; }
using ushort2v = unsigned short __attribute__((ext_vector_type(2)));

// Largest of fp16 numbers that are not negative, two at a time: their bit patterns order like the numbers.
__device__ __forceinline__ uint32_t max_bits(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2v, a), __builtin_bit_cast(ushort2v, b)));
}
__device__ __forceinline__ float larger_half(uint32_t a) {
  const half2v h = as_half2(a);
  return fmaxf((float)h[0], (float)h[1]);
}
// Over the eight lanes (l & ~7) .. (l | 7): used by the single-row path, where the eight tokens a
// lane group shares are spread over eight lanes.
__device__ __forceinline__ float octet_max(float x) {
  x = fmaxf(x, __shfl_xor(x, 1));
  x = fmaxf(x, __shfl_xor(x, 2));
  return fmaxf(x, __shfl_xor(x, 4));
}
__device__ __forceinline__ float octet_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x + __shfl_xor(x, 4);
}
// Lane i of a 16-lane row takes `src` of lane i - K (K = 1..15); lanes i < K keep `old`.
template <int K>
__device__ __forceinline__ uint32_t row_shr_keep(uint32_t old, uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, 0x110 + K, 0xF, 0xF, false);
}
// Lane i of a 16-lane row takes `src` of lane i + K; lanes past the end of the row take 0.
template <int K>
__device__ __forceinline__ uint32_t row_shl_zero(uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)src, 0x100 + K, 0xF, 0xF, true);
}


// ------------------------------------------------------------------------------------------------
// Query rows on the 16 columns of an MFMA tile.  A tile carries 16 or 8 query rows (its mode M):
//   M = 16  column c = row c.  The remainder of q*S (see the file header) is a second operand that is
//           accumulated into the same result.
//   M = 8   columns c and c + 8 = row c: q*S in the first, its remainder in the second; one DPP add
//           recombines the scores, after which both columns hold the same and do the same work.
// Either way a lane owns the 8 tokens of its lane group for the query row of its column.
// ------------------------------------------------------------------------------------------------
struct Lane {
  int rho, g;   // MFMA column and lane group
  __device__ __forceinline__ Lane() {
    const int lane = threadIdx.x & 63;
    rho = lane & 15;
    g = lane >> 4;
  }
  template <int M>
  __device__ __forceinline__ int row() const { return rho & (M - 1); }          // row of the tile this column serves
  template <int M>
  __device__ __forceinline__ bool remainder() const { return M == 8 && rho >= 8; }   // column holds the remainder of q*S
};

template <int K>
__device__ __forceinline__ float ror_in_row(float x) {   // value of lane (l + K) mod 16 of the same 16-lane row
  const int v = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0x120 + K, 0xF, 0xF, true));
}

// The scores of this lane's eight tokens from the two MFMA results of a block (a0: tokens 0..15,
// a1: 16..31; element jj of either is token 4g + jj of that half).
template <int M>
__device__ __forceinline__ void tile_scores(const float4v& a0, const float4v& a1, float (&x)[8]) {
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    x[jj] = M == 16 ? a0[jj] : a0[jj] + ror_in_row<8>(a0[jj]);
    x[4 + jj] = M == 16 ? a1[jj] : a1[jj] + ror_in_row<8>(a1[jj]);
  }
}

// ------------------------------------------------------------------------------------------------
// Online softmax with a reference that moves rarely.  A row keeps a reference exponent m (log2 units)
// and everything it accumulates - sum l, zero-point term z, output o - is relative to it:
// p = 2^(score - m).  m does not have to be the largest score: any reference works as long as p fits
// its formats, and the merge of the partials is indifferent to it.  So m is only raised when a score
// of the wave exceeds it by more than kTau (p > 2^kTau), and is then put kLift below the largest score
// of the row.  (m also carries the exponent e of the value scales, see raise_scale_reference: the bounds
// here are on p * 2^e.)  After the first blocks of a chunk that practically never happens again, so the main
// path of a block has no cross-lane reduction and no rescaling of the accumulators - with 20 query
// rows per wave the classic running maximum took the rescaling path in nearly every second block.
// p <= 2^kTau = 256 and p * S <= 512 (S: see raise_scale_reference) stay far inside fp16.
// ------------------------------------------------------------------------------------------------
constexpr float kTau = 8.0f;
constexpr float kLift = 2.0f;

template <int NRT>
struct RowState {
  float m[NRT];        // reference exponent of the row (includes e)
  float e;             // floor(log2) of the largest value scale met so far by the wave; 0 in the buffer chunk
  float s_limit;       // 2^(e + 1): a larger value scale raises e
  float l[NRT];        // running sum of p over this lane's tokens
  float z[NRT];        // running sum of p * zero-point over this lane's tokens
  float4v o[NRT][8];   // O^T accumulators: tile n, element jj -> channel 8*(4*g + jj) + n
  __device__ __forceinline__ void reset(float e0, float limit0) {
    e = e0;
    s_limit = limit0;
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      m[rt] = kNegBig, l[rt] = 0.f, z[rt] = 0.f;
#pragma unroll
      for (int n = 0; n < 8; ++n) o[rt][n] = (float4v){0.f, 0.f, 0.f, 0.f};
    }
  }
};

// Rescaling of an output accumulator on one of the rare paths.  PIN: the kernel keeps its accumulators
// in the accumulation registers, where the matrix cores update them in place; the empty statement
// says that the value is there when the rare path begins, so the copy to the arithmetic registers
// that the multiplication needs is made here and not ahead of the branch, in every block.
template <bool PIN>
__device__ __forceinline__ void scale_acc(float4v& o, float alpha) {
  if constexpr (PIN) asm volatile("" : "+a"(o));
  o *= alpha;
}

__device__ __forceinline__ float max_of(const float (&v)[8]) {
  return fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
}

// The rare path of a tile.  arg: the exponents score - m of this lane's tokens, relative to the row's
// present reference m = (score level) + e.  Raises the score level to kLift below the row's largest
// score if that is higher than the present one, rescales what the row has accumulated and rebases the
// exponents.
template <bool PIN, int NRT>
__device__ __forceinline__ void raise_reference(RowState<NRT>& st, int rt, float (&arg)[8]) {
  const float top = group_max(max_of(arg));
  const float delta = fmaxf(top + st.e - kLift, 0.f);
  const float alpha = __builtin_amdgcn_exp2f(-delta);
  st.m[rt] += delta;
  st.l[rt] *= alpha;
  st.z[rt] *= alpha;
#pragma unroll
  for (int n = 0; n < 8; ++n) scale_acc<PIN>(st.o[rt][n], alpha);
#pragma unroll
  for (int j = 0; j < 8; ++j) arg[j] -= delta;
}

// The first reference of a row, from the scaled scores s of the first block the wave sees (nothing
// has been accumulated yet).  A row whose tokens are all masked keeps "no reference".
template <int NRT>
__device__ __forceinline__ void first_reference(RowState<NRT>& st, int rt, const float (&s)[8]) {
  st.m[rt] = fmaxf(group_max(max_of(s)) - kLift + st.e, kNegBig);
}

// The row reference carries, on top of the score part, the exponent e of the largest value scale S
// met so far, so that p * S, which enters the second contraction as fp16, keeps its bits however
// small or large the values are (S / 2^e < 2 for the largest S).  Called with this lane group's largest
// scale of the block after the block's probabilities exist and before they are used: when a scale of
// the wave exceeds 2^(e+1), e is raised and everything that carries the old reference, the block's
// probabilities included, is scaled down by the same power of two.
template <bool PIN, int NRT, typename ScaleP>
__device__ __forceinline__ void raise_scale_reference(RowState<NRT>& st, float smax, ScaleP&& scale_p) {
  if (__any(smax > st.s_limit)) {
    const float s_all = group_max(smax);   // the same in every lane: lanes of one group share their tokens
    const uint32_t ebits = __builtin_bit_cast(uint32_t, s_all) & 0x7f800000u;   // 2^floor(log2 s_all)
    const float e_new = (float)((int)(ebits >> 23) - 127);
    const float delta = e_new - st.e;                     // > 0
    const float alpha = __builtin_amdgcn_exp2f(-delta);   // a power of two: exact
    st.e = e_new;
    st.s_limit = 2.0f * __builtin_bit_cast(float, ebits);
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      st.m[rt] += delta;
      st.l[rt] *= alpha;
      st.z[rt] *= alpha;
#pragma unroll
      for (int n = 0; n < 8; ++n) scale_acc<PIN>(st.o[rt][n], alpha);
    }
    scale_p(alpha);
  }
}

// Largest of the eight fp16 value scales of a lane group (positive numbers; packed maxima).
__device__ __forceinline__ float max_scale(const u32x4& d) {
  const half2v a = __builtin_elementwise_max(as_half2(d[0]), as_half2(d[1]));
  const half2v b = __builtin_elementwise_max(as_half2(d[2]), as_half2(d[3]));
  const half2v c = __builtin_elementwise_max(a, b);
  return (float)__builtin_elementwise_max(c[0], c[1]);
}

// One 32-token block of a kv-head with a single query row (multi-head attention, one decode query).
// After the first contraction the row's 32 scores sit eight per lane in the four lanes of column 0
// and the other 60 lanes would repeat the whole softmax on columns nobody reads.  Instead the eight
// scores of lane (0, g) are dealt out to lanes (k, g), k = 0..7 (lanes 8..15 mirror them), so that
// every lane carries ONE token: one exponential, one value scale, one zero-point per lane and block.
// The probabilities go back as fp16 pairs, which leaves the second operand of the value contraction
// complete in lane (0, g) - the only column whose result is kept.  Sums (l, z) stay per lane and are
// folded over the eight lanes once, before the partial is written.
// raw: this lane's eight combined scores (meaningful in column 0); s_bits, z_bits: fp16 scale and
// zero-point of token tile_token(g, rho & 7); first: the wave's first block.  Returns the lane's operand of the value contraction.
template <bool VERIFY>
__device__ __forceinline__ half8 single_row_block(RowState<1>& st, const float (&raw)[8], float mul, float bias,
                                                  uint32_t s_bits, uint32_t z_bits, int rho, bool first) {
  auto bits = [](float f) { return __builtin_bit_cast(uint32_t, f); };
  uint32_t w = bits(raw[0]);
  w = row_shr_keep<1>(w, bits(raw[1]));
  w = row_shr_keep<2>(w, bits(raw[2]));
  w = row_shr_keep<3>(w, bits(raw[3]));
  w = row_shr_keep<4>(w, bits(raw[4]));
  w = row_shr_keep<5>(w, bits(raw[5]));
  w = row_shr_keep<6>(w, bits(raw[6]));
  w = row_shr_keep<7>(w, bits(raw[7]));
  w = (uint32_t)__builtin_amdgcn_update_dpp((int)w, (int)w, 0x118, 0xF, 0xC, false);   // lanes 8..15 <- lanes 0..7
  const float x = __builtin_bit_cast(float, w);

  const float base = bias * mul;
  if (first) st.m[0] = group_max(octet_max(__builtin_fmaf(x, mul, base))) - kLift + st.e;   // see first_reference
  float arg = __builtin_fmaf(x, mul, base - st.m[0]);
  if (__any(arg > kTau - st.e)) {   // see raise_reference
    const float delta = fmaxf(group_max(octet_max(arg)) + st.e - kLift, 0.f);
    const float alpha = __builtin_amdgcn_exp2f(-delta);
    st.m[0] += delta;
    st.l[0] *= alpha;
    st.z[0] *= alpha;
#pragma unroll
    for (int n = 0; n < 8; ++n) st.o[0][n] *= alpha;
    arg -= delta;
  }
  float p = __builtin_amdgcn_exp2f(arg);

  const float sv = (float)__builtin_bit_cast(_Float16, (uint16_t)s_bits);
  const float zv = (float)__builtin_bit_cast(_Float16, (uint16_t)z_bits);
  raise_scale_reference<false>(st, octet_max(sv), [&](float alpha) { p *= alpha; });
  st.l[0] += p;
  st.z[0] = __builtin_fmaf(p, VERIFY ? __builtin_fmaf(-0.5f, sv, zv) : zv, st.z[0]);
  _Float16 h = (_Float16)(p * sv);
  if (!VERIFY) h = h * (_Float16)((rho & 2) ? 0.0625f : 1.0f);   // elements 2,3,6,7 of the operand: see the value unpacking
  const uint32_t hb = __builtin_bit_cast(uint16_t, h);
  const uint32_t pair = hb | (row_shl_zero<1>(hb) << 16);
  const u32x4 pw = {pair, row_shl_zero<2>(pair), row_shl_zero<4>(pair), row_shl_zero<6>(pair)};
  return as_half8(pw);
}

// Tile rt of a wave that carries NRT tiles: all but the last are full (16 rows), the last has mode TAIL.
template <int NRT, int TAIL>
constexpr int mode_of(int rt) { return rt == NRT - 1 ? TAIL : 16; }

template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

// Writes the partial (m, l, o) of every row of the wave.  o_scale: factor on the raw accumulators.
template <int NRT, int TAIL>
__device__ __forceinline__ void write_partial(const AttnArgs& a, RowState<NRT>& st, int b, int kvh, int row0,
                                              int split, float o_scale) {
  const Lane L;
  const int n_split = a.n_split_q + a.n_split_b;
  static_for<NRT>([&](auto RT) {
    constexpr int rt = decltype(RT)::value;
    constexpr int M = mode_of<NRT, TAIL>(rt);
    const float l = group_sum(st.l[rt]);
    const float z = group_sum(st.z[rt]);
    const int row = row0 + 16 * rt + L.row<M>();
    const bool writer = L.rho < M && row < a.n_rows;
    const int qi = row / a.rep, head = kvh * a.rep + row % a.rep;
    const int64_t r = (((int64_t)b * a.nq + qi) * a.n_q_heads + head) * n_split + split;
    float* po = a.ws_o + r * kD;
    if (writer) {
#pragma unroll
      for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) po[8 * (4 * L.g + jj) + n] = __builtin_fmaf(st.o[rt][n][jj], o_scale, z);
    }
    if (writer && L.g == 0) {
      a.ws_ml[2 * r] = st.m[rt];
      a.ws_ml[2 * r + 1] = l;
    }
  });
}

// ------------------------------------------------------------------------------------------------
// A chunk of the quantized region: a contiguous range of 128-token groups of one unit.
//
// The wave walks its chunk in 32-token blocks.  Each block is eight (draft: four) 1 KB plane loads
// and four 16-byte metadata loads per lane, straight into registers; the loads of block i+1 are in
// flight while block i is computed (register double buffering).  The loop is unrolled over the four
// blocks of a group so that the query operand of the NEXT group (q*S, needs that group's key
// metadata) is built one MFMA k-step per block and no bubble appears at group boundaries.
// ------------------------------------------------------------------------------------------------
//
// Which groups a wave walks: a fixed contiguous range (split `split` of n_split_q of the unit), or -
// DYN - groups [g_base, g_base + g_count) handed out one at a time through the counter `queue` that
// the waves of a workgroup share in LDS (first_claim: the value this wave already drew).  The
// pipeline looks two groups ahead (block prefetch, key metadata of the next group), so the wave
// always holds the group it computes and the next two it has drawn.
template <int NRT, int TAIL, bool VERIFY, bool SINGLE, bool PAGED, bool DYN = false>
__device__ __forceinline__ void quant_chunk(const AttnArgs& a, int unit, int b, int kvh, int row0, int split,
                                            int* queue = nullptr, int g_base = 0, int g_count = 0, int first_claim = 0) {
  static_assert(!SINGLE || (NRT == 1 && TAIL == 8), "the single-row path is a variant of the one-tile kernel");
  constexpr bool kTwoWaves = NRT == 1 && TAIL != 16;   // room for two waves per SIMD: at most 256 registers, none of them accumulation registers
  constexpr bool PIN = !kTwoWaves;
  const Lane L;
  const int lane = threadIdx.x & 63, rho = L.rho, g = L.g;
  const int n_groups = a.len.n_quant[b] / kG;
  int first = 0, n_local = 0;
  int gq[3] = {-1, -1, -1};   // DYN: the group being computed and the two drawn after it (-1: none left)
  auto draw = [&]() -> int {
    int v = 0;
    if (lane == 0) v = atomicAdd(queue, 1);
    v = __builtin_amdgcn_readfirstlane(v);
    return v < g_count ? g_base + v : -1;
  };
  // A wave holds the group it computes and the next one (blocks and key metadata are asked for one group
  // ahead); with a group table also the one after, whose table entry must be on its way a group earlier.
  constexpr bool kThreeHeld = PAGED;
  if constexpr (DYN) {
    gq[0] = first_claim < g_count ? g_base + first_claim : -1;
    gq[1] = gq[0] >= 0 ? draw() : -1;
    if (kThreeHeld) gq[2] = gq[1] >= 0 ? draw() : -1;
    n_local = gq[0] >= 0 ? 1 : 0;
  } else {
    first = (int)((int64_t)split * n_groups / a.n_split_q);
    n_local = (int)((int64_t)(split + 1) * n_groups / a.n_split_q) - first;
  }

  // Powers of two folded out of the operands (see file header).
  //   draft : code operand carries 2^-24 (elements 0,1,4,5) or 2^-20 (elements 2,3,6,7); the other
  //           operand of either contraction takes 2^-4 at the latter
  //   verify: code operand carries 2^-24 and the codes are 16*C_U + C_L + 8 in units of S/16
  constexpr float kKeyPos = VERIFY ? 1.0f : 0.0625f;             // factor on q at elements 2,3,6,7
  constexpr float kKeyRaw = VERIFY ? 1048576.0f : 16777216.0f;   // score = raw * kKeyRaw * c0
  constexpr float kOutRaw = VERIFY ? 1048576.0f : 16777216.0f;   // out = rawO * kOutRaw + sum p*Zeff

  RowState<NRT> st;
  st.reset(-40.f, 0x1p-39f);   // e below every value scale (>= 2^-24): the first block raises it
  if (n_local <= 0) {
    write_partial<NRT, TAIL>(a, st, b, kvh, row0, split, kOutRaw);
    return;
  }

  // Start of chunk-local block j in the upper / lower array.  Contiguous units: blocks follow each
  // other; with a group table every 128-token group (four blocks) is looked up.
  // The table entries of the three groups the pipeline holds (the one being computed, the next, the one
  // after) are asked for when a group enters the pipeline, a whole group before its first address is
  // formed, and are only waited for there: a lookup at the point of use would stop the wave for a trip to
  // memory eight times per group.
  constexpr bool paged = PAGED;   // (a kernel of its own: the table entries carried from round to round cost the others a wait)
  const int64_t blk0 = ((int64_t)unit * (a.q_cap / kG) + first) * (kG / kBlkTok);
  int place[3] = {0, 0, 0};   // paged: where those three groups lie (the same in every lane)
  int cur_lg = 0;             // fixed ranges: chunk-local number of the group being computed
  auto look_up = [&](int gi) -> int { return a.group_table[(int64_t)unit * (a.q_cap / kG) + gi]; };
  auto held = [&](int k) -> int64_t {   // place[k], k in 0..2
    const int v = k == 0 ? place[0] : k == 1 ? place[1] : place[2];
    return (int64_t)__builtin_amdgcn_readfirstlane(v);
  };
  auto block_index = [&](int j) -> int64_t {
    if constexpr (DYN) {   // j: 0..3 the current group, 4..7 the next; none left: the current one
      int sel = j >> 2;
      if (gq[sel] < 0) sel = 0;
      return (paged ? held(sel) : (int64_t)unit * (a.q_cap / kG) + gq[sel]) * (kG / kBlkTok) + (j & 3);
    } else {
      return paged ? held((j >> 2) - cur_lg) * (kG / kBlkTok) + (j & 3) : blk0 + j;
    }
  };
  if (paged) {
    if constexpr (DYN) {
#pragma unroll
      for (int k = 0; k < 3; ++k)
        if (gq[k] >= 0) place[k] = look_up(gq[k]);
    } else {
#pragma unroll
      for (int k = 0; k < 3; ++k) place[k] = look_up(first + min(k, n_local - 1));
    }
  }
  const int k_off = kOffK + rho * 64 + 16 * g;   // key rows rho and 16 + rho, channels 32g ..
  const int v_off = kOffV + 16 * lane;           // value tile, two halves of 1 KB
  const int m_off = 16 * g;                      // metadata: eight fp16 of lane group g

  // One 32-token block of operands.
  struct Blk {
    u32x4 kU[2], kL[2], vU[2], vL[2];   // two 16-token key tiles, two halves of the value tile
    u32x4 vS, vZ;                       // value S / Z of this lane group's eight tokens
  };
  // loads of block j (chunk-local); past the end of the chunk the last block is re-read and never used
  auto load_block = [&](Blk& d, int j) {
    const int jc = DYN ? j : min(j, 4 * n_local - 1);
    const int64_t bj = block_index(jc);
    const __amdgpu_buffer_rsrc_t u = block_resource(a.upper + bj * kUpperBlk, kUpperBlk);
    d.kU[0] = ldb128_stream(u, k_off);
    d.kU[1] = ldb128_stream(u, k_off + 1024);
    d.vU[0] = ldb128_stream(u, v_off);
    d.vU[1] = ldb128_stream(u, v_off + 1024);
    if (SINGLE) {   // this lane's own token only
      d.vS[0] = ldb16_stream(u, kOffVS + m_off + 2 * (rho & 7));
      d.vZ[0] = ldb16_stream(u, kOffVZ + m_off + 2 * (rho & 7));
    } else {
      d.vS = ldb128_stream(u, kOffVS + m_off);
      d.vZ = ldb128_stream(u, kOffVZ + m_off);
    }
    if (VERIFY) {
      const __amdgpu_buffer_rsrc_t l = block_resource(a.lower + bj * kLowerBlk, kLowerBlk);
      d.kL[0] = ldb128_stream(l, k_off);
      d.kL[1] = ldb128_stream(l, k_off + 1024);
      d.vL[0] = ldb128_stream(l, v_off);
      d.vL[1] = ldb128_stream(l, v_off + 1024);
    }
  };
  // Blocks in flight ahead of the one being computed.  With a single block ahead the bytes a wave
  // keeps in flight, divided by the memory latency under load, cap the bandwidth below what the
  // memory delivers; the draft kernel has the registers for a second one (three of the four named
  // buffers are live at any time).
  constexpr int kAhead = (!VERIFY && kTwoWaves) ? 2 : 1;
  Blk bufA, bufB, bufC, bufD;
  // Key S / Z of the four k-steps of the NEXT group, asked for at the top of a round and used from its
  // second block on.  (Fetched with the blocks instead, two of the four crossed the end of the round in
  // registers that the compiler would not keep in place: it copied them there, behind a wait for every
  // load in flight, once per group.)
  u32x4 nkS[4], nkZ[4];
  auto load_next_meta = [&](int lg) {
    const uint8_t* nb = a.upper + block_index(DYN ? 4 : min(lg + 1, n_local - 1) * 4) * kUpperBlk;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      nkS[s4] = ldg128_stream(nb + s4 * kUpperBlk + kOffKS + m_off);
      nkZ[s4] = ldg128_stream(nb + s4 * kUpperBlk + kOffKZ + m_off);
    }
  };
  // Everything the first group needs first is requested before anything is waited for: as many of its
  // blocks as the loop keeps in flight, and its key metadata.  (All four blocks at once, where the
  // registers allow it, put 35 MB of requests in front of the memory at the start of a 128k-context
  // launch: the median wave then holds its first block after 6.4 us instead of 4.4 us, the waves served
  // last start 6 us behind the first, and the draft call is 0.2 - 0.5 us longer at 32k and 128k context.)
  load_block(bufA, 0);
  if (kAhead == 2) load_block(bufB, 1);
  const uint8_t* ub = a.upper + block_index(0) * kUpperBlk;   // the four blocks of a group are adjacent
  u32x4 ks0[4], kz0[4];
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4) {
    ks0[s4] = ldg128_stream(ub + s4 * kUpperBlk + kOffKS + m_off);
    kz0[s4] = ldg128_stream(ub + s4 * kUpperBlk + kOffKZ + m_off);
  }

  // Queries of this lane's column: channels 32*g + 8*s + operand order.  Each row is scaled by a power
  // of two so that max|q| <= 1 (the key scales are lifted below 2^15, see next_lift: q*S cannot overflow
  // fp16 whatever the inputs are); the power goes into the row's score multiplier.  Elements 2,3,6,7 also take the code operand's 2^-4.
  half2v qv[NRT][16];
  float mul[NRT];
  static_for<NRT>([&](auto RT) {
    constexpr int rt = decltype(RT)::value;
    constexpr int M = mode_of<NRT, TAIL>(rt);
    const int row = row0 + 16 * rt + L.row<M>();
    const bool valid = row < a.n_rows;
    const int rowc = valid ? row : 0;
    const int qi = rowc / a.rep, head = kvh * a.rep + rowc % a.rep;
    const _Float16* qp = a.q + (((int64_t)b * a.nq + qi) * a.n_q_heads + head) * kD + 32 * g;
    u32x4 w[4];
    float amax = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const half8 h = to_operand_order(as_half8(ldg128(qp + 8 * s)));
      w[s] = as_u32x4(h);
#pragma unroll
      for (int e = 0; e < 8; ++e) amax = fmaxf(amax, __builtin_fabsf((float)h[e]));
    }
    amax = group_max(amax);
    // 2^-e with 2^e >= max|q| (e = 0 for an all-zero row); exact in fp16 and fp32
    const int e = amax > 0.f ? max(-14, (int)((__builtin_bit_cast(uint32_t, amax) >> 23) & 0xff) - 126) : 0;
    const float down = __builtin_bit_cast(float, (uint32_t)(127 - e) << 23);
    mul[rt] = a.c0 * kKeyRaw * __builtin_bit_cast(float, (uint32_t)(127 + e) << 23);
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        half2v h = as_half2(valid ? w[s][r] : 0u);
        h = h * (_Float16)(down * ((r & 1) ? kKeyPos : 1.0f));
        qv[rt][4 * s + r] = h;
      }
  });

  // Query operand of the current group (qb, cin) and, built one k-step per block, of the next one.
  // q*S is split exactly into fp16(q*S) and the fp16 remainder q*S - fp16(q*S): two operands
  // accumulated into the same MFMA result for a tile of 16 rows, two columns of one operand otherwise.
  // The scales of a group are first lifted by the power of two 2^fs that brings the largest of them, over all
  // channels, into [2^14, 2^15): exact, and with |q| <= 1 the products stay inside fp16 while the remainder keeps
  // its bits however small the keys' spread is.  gmul, the group's score multiplier, takes the lift back.
  half8 qb[NRT][2][4], qbn[NRT][2][4];
  float cin[NRT], gmul[NRT], acc_a[NRT], acc_b[NRT], acc_sa[NRT], acc_sb[NRT];
  int fs_n = 0;
  _Float16 up_n = (_Float16)1.0f;
  auto next_lift = [&](const u32x4 (&S)[4]) {   // S: the key scales of this lane's 32 channels; the four lane groups cover all 128
    uint32_t sm = 0u;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
      for (int r = 0; r < 4; ++r) sm = max_bits(sm, S[s4][r]);
    fs_n = min(14 - max(exponent_of(group_max(larger_half(sm))), -24), 15);
    up_n = (_Float16)pow2(fs_n);
  };
  auto prep_reset = [&]() {
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) acc_a[rt] = acc_b[rt] = acc_sa[rt] = acc_sb[rt] = 0.f;
  };
  auto prep_kstep = [&](auto S, u32x4 sw, u32x4 zw) {   // sw, zw: key S / Z of channels 32g + 8s.., operand order
    constexpr int s = decltype(S)::value;
    half2v lifted[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) lifted[r] = as_half2(sw[r]) * up_n;
    static_for<NRT>([&](auto RT) {
      constexpr int rt = decltype(RT)::value;
      constexpr int M = mode_of<NRT, TAIL>(rt);
      u32x4 out, out_lo;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const half2v qh = qv[rt][4 * s + r], sh = as_half2(sw[r]), zh = as_half2(zw[r]);
        const half2v hi = qh * lifted[r];
        const half2v lo = __builtin_elementwise_fma(qh, lifted[r], -hi);
        if (M == 16) {
          out[r] = as_u32(hi);
          out_lo[r] = as_u32(lo);
        } else {
          out[r] = L.remainder<M>() ? as_u32(lo) : as_u32(hi);
        }
        if (r & 1) {
          acc_b[rt] = __builtin_amdgcn_fdot2(qh, zh, acc_b[rt], false);
          if (VERIFY) acc_sb[rt] = __builtin_amdgcn_fdot2(qh, sh, acc_sb[rt], false);
        } else {
          acc_a[rt] = __builtin_amdgcn_fdot2(qh, zh, acc_a[rt], false);
          if (VERIFY) acc_sa[rt] = __builtin_amdgcn_fdot2(qh, sh, acc_sa[rt], false);
        }
      }
      qbn[rt][0][s] = as_half8(out);
      if (M == 16) qbn[rt][1][s] = as_half8(out_lo);
    });
  };
  auto prep_commit = [&]() {   // sum_d q_d * Zeff_d, Zeff = Z (draft) or Z - S/2 (verify: codes carry +8 lower steps)
    static_for<NRT>([&](auto RT) {
      constexpr int rt = decltype(RT)::value;
      constexpr int M = mode_of<NRT, TAIL>(rt);
      float bias = __builtin_fmaf(acc_b[rt], 1.0f / kKeyPos, acc_a[rt]);
      if (VERIFY) bias -= 0.5f * __builtin_fmaf(acc_sb[rt], 1.0f / kKeyPos, acc_sa[rt]);
      bias = group_sum(bias);
      cin[rt] = bias * (1.0f / kKeyRaw) * pow2(fs_n);   // added to the raw scores inside the softmax step
      gmul[rt] = mul[rt] * pow2(-fs_n);
      if (SINGLE) cin[rt] = __shfl(cin[rt], lane & 48);   // every lane works on the one row of column 0
#pragma unroll
      for (int h = 0; h < (M == 16 ? 2 : 1); ++h)
#pragma unroll
        for (int s = 0; s < 4; ++s) qb[rt][h][s] = qbn[rt][h][s];
    });
    prep_reset();
  };

  bool fresh = true;   // the wave's first block sets the rows' references
  auto compute_block = [&](const Blk& d, auto P) {
    constexpr int p = decltype(P)::value;
    // ---- scores: S^T[token, column] = codes x q ----
    float x[NRT][8];   // raw scores of this lane's eight tokens; later their exponents, then their probabilities
    {
      half8 ka[2][4];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < 4; ++s) ka[t][s] = VERIFY ? unpack8(d.kU[t][s], d.kL[t][s]) : unpack4(d.kU[t][s]);
      static_for<NRT>([&](auto RT) {
        constexpr int rt = decltype(RT)::value;
        constexpr int M = mode_of<NRT, TAIL>(rt);
        float4v acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          acc[t] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][s], qb[rt][0][s], acc[t], 0, 0, 0);
            if (M == 16) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][s], qb[rt][1][s], acc[t], 0, 0, 0);
          }
        }
        tile_scores<M>(acc[0], acc[1], x[rt]);
      });
    }
    // the next group's query operand, spread over the blocks that follow the arrival of its metadata
    if constexpr (p == 1) {
      next_lift(nkS);
      prep_kstep(std::integral_constant<int, 0>{}, nkS[0], nkZ[0]);
    }
    if constexpr (p == 2) {
      prep_kstep(std::integral_constant<int, 1>{}, nkS[1], nkZ[1]);
      prep_kstep(std::integral_constant<int, 2>{}, nkS[2], nkZ[2]);
    }
    if constexpr (p == 3) prep_kstep(std::integral_constant<int, 3>{}, nkS[3], nkZ[3]);
    half8 pb[NRT];
    if constexpr (SINGLE) {
      pb[0] = single_row_block<VERIFY>(st, x[0], gmul[0], cin[0], d.vS[0], d.vZ[0], rho, p == 0 && fresh);
    } else {
      // ---- probabilities relative to the rows' references (see above) ----
      float base[NRT];
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) base[rt] = cin[rt] * gmul[rt];
      if (p == 0 && fresh) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          float s[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) s[j] = __builtin_fmaf(x[rt][j], gmul[rt], base[rt]);
          first_reference(st, rt, s);
        }
      }
      const float limit = kTau - st.e;   // exponents are short of the scores by e
      bool high = false;
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        const float shift = base[rt] - st.m[rt];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[rt][j] = __builtin_fmaf(x[rt][j], gmul[rt], shift);   // the exponent score - m
        high |= max_of(x[rt]) > limit;
      }
      if (__any(high)) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) raise_reference<PIN>(st, rt, x[rt]);
      }
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          x[rt][j] = __builtin_amdgcn_exp2f(x[rt][j]);   // the probability
          sum += x[rt][j];
        }
        st.l[rt] += sum;
      }

      // ---- probabilities x value scale -> B operand; zero-point term ----
      raise_scale_reference<PIN>(st, max_scale(d.vS), [&](float alpha) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
          for (int j = 0; j < 8; ++j) x[rt][j] *= alpha;
      });
      // The scales and zeros enter as the fp16 numbers they are (mixed-precision multiply-adds: no conversion
      // of its own, and the product comes out as the fp16 half of the operand word), products in binary32.
      const half8 sv = as_half8(d.vS), zv = as_half8(d.vZ);
      float zeff[8];
      if (VERIFY) {
#pragma unroll
        for (int j = 0; j < 8; ++j) zeff[j] = __builtin_fmaf(-0.5f, (float)sv[j], (float)zv[j]);
      }
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        float zs = 0.f;
        half8 ph;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          zs = __builtin_fmaf(x[rt][j], VERIFY ? zeff[j] : (float)zv[j], zs);
          ph[j] = (_Float16)__builtin_fmaf(x[rt][j], (float)sv[j], 0.f);
        }
        st.z[rt] += zs;
        if (!VERIFY) {   // the words whose codes sit four bits higher in their half (odd words) take 2^-4
          u32x4 pw = as_u32x4(ph);
          pw[1] = as_u32(as_half2(pw[1]) * (_Float16)0.0625f);
          pw[3] = as_u32(as_half2(pw[3]) * (_Float16)0.0625f);
          ph = as_half8(pw);
        }
        pb[rt] = ph;
      }
    }

    // ---- O^T[channel, column] += codes^T x p ----
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const half8 va = VERIFY ? unpack8(d.vU[n >> 2][n & 3], d.vL[n >> 2][n & 3]) : unpack4(d.vU[n >> 2][n & 3]);
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt)
        st.o[rt][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pb[rt], st.o[rt][n], 0, 0, 0);
    }
    if (p == 3) prep_commit();
    if (p == 0) fresh = false;
  };

  // the first group's query operand from the metadata requested at the start
  prep_reset();
  next_lift(ks0);
  prep_kstep(std::integral_constant<int, 0>{}, ks0[0], kz0[0]);
  prep_kstep(std::integral_constant<int, 1>{}, ks0[1], kz0[1]);
  prep_kstep(std::integral_constant<int, 2>{}, ks0[2], kz0[2]);
  prep_kstep(std::integral_constant<int, 3>{}, ks0[3], kz0[3]);
  prep_commit();

  for (int lg = 0; DYN ? gq[0] >= 0 : lg < n_local; ++lg) {
    const int j = DYN ? 0 : 4 * lg;   // DYN: block numbers are relative to the current group
    load_next_meta(lg);
    if (kAhead == 2) {
      load_block(bufC, j + 2);
      compute_block(bufA, std::integral_constant<int, 0>{});
      load_block(bufD, j + 3);
      compute_block(bufB, std::integral_constant<int, 1>{});
      load_block(bufA, j + 4);
      compute_block(bufC, std::integral_constant<int, 2>{});
      load_block(bufB, j + 5);
      compute_block(bufD, std::integral_constant<int, 3>{});
    } else {
      load_block(bufB, j + 1);
      compute_block(bufA, std::integral_constant<int, 0>{});
      load_block(bufA, j + 2);
      compute_block(bufB, std::integral_constant<int, 1>{});
      load_block(bufB, j + 3);
      compute_block(bufA, std::integral_constant<int, 2>{});
      load_block(bufA, j + 4);
      compute_block(bufB, std::integral_constant<int, 3>{});
    }
    if constexpr (DYN) {
      gq[0] = gq[1];
      if (kThreeHeld) {
        gq[1] = gq[2];
        gq[2] = gq[1] >= 0 ? draw() : -1;
      } else {
        gq[1] = gq[0] >= 0 ? draw() : -1;
      }
    }
    cur_lg = lg + 1;
    if (paged) {
      place[0] = place[1];
      place[1] = place[2];
      if constexpr (DYN) {
        if (gq[2] >= 0) place[2] = look_up(gq[2]);
      } else {
        place[2] = look_up(first + min(lg + 3, n_local - 1));
      }
    }
  }
  if constexpr (SINGLE) {   // one token per lane: the row's sums are spread over eight lanes
    st.l[0] = octet_sum(st.l[0]);
    st.z[0] = octet_sum(st.z[0]);
    write_partial<1, 16>(a, st, b, kvh, row0, split, kOutRaw);   // column 0 alone holds the row: nothing to add up
    return;
  }
  write_partial<NRT, TAIL>(a, st, b, kvh, row0, split, kOutRaw);
}

// ------------------------------------------------------------------------------------------------
// A chunk of the full-precision buffer: a range of its 32-token blocks (two for a decode-time
// buffer, many when the buffer is long, e.g. a cache that keeps every token in fp16).  Keys are read
// straight into the A operand; the value rows are transposed through LDS because the matrix cores
// need eight tokens of one channel per lane while the buffer is stored token-major.  The next
// block's keys and values are in flight while the current one is computed.  fp16 queries and keys
// need no remainder part, so every column of a tile is a query row here (NRT tiles of 16 rows).
// ------------------------------------------------------------------------------------------------
constexpr int kVtStride = 40;   // halfs per LDS row: 32 tokens + padding, keeps 8-byte reads aligned

// A transpose tile is written and read by the lanes of ONE wave only.  The LDS executes a wave's
// instructions in order, so all that is needed between its writes and its reads is that neither the
// compiler nor the wave's own outstanding-operation counter lets them pass each other; a workgroup
// barrier would be wrong where the waves of a workgroup work on unrelated items.
__device__ __forceinline__ void wave_lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
constexpr float kBufP = 128.0f;   // p <= 2^kTau: p * kBufP stays inside fp16

template <int NRT>
__device__ __forceinline__ void buffer_chunk(const AttnArgs& a, int unit, int b, int kvh, int row0, int split,
                                             _Float16 (*vt)[kVtStride]) {
  const int lane = threadIdx.x & 63, rho = lane & 15, g = lane >> 4;
  const int nb = a.len.n_buf[b];
  // the buffer's 32-token blocks are dealt out evenly to its n_split_b chunks
  const int n_blk = (nb + 31) >> 5, piece = split - a.n_split_q;
  const int blk0 = (int)((int64_t)piece * n_blk / a.n_split_b);
  const int blk1 = (int)((int64_t)(piece + 1) * n_blk / a.n_split_b);

  half8 qb[NRT][4];
  int vis[NRT];   // buffer tokens [0, vis) are visible to this lane's query (causal among the nq queries)
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int row = row0 + 16 * rt + rho;
    const bool valid = row < a.n_rows;
    const int rowc = valid ? row : 0;
    const int qi = rowc / a.rep, head = kvh * a.rep + rowc % a.rep;
    const _Float16* qp = a.q + (((int64_t)b * a.nq + qi) * a.n_q_heads + head) * kD + 8 * g;
    vis[rt] = valid ? nb - a.nq + qi + 1 : 0;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4 w = ldg128(qp + 32 * s);
      if (!valid) w = (u32x4){0u, 0u, 0u, 0u};
      qb[rt][s] = as_half8(w);
    }
  }
  RowState<NRT> st;
  st.reset(0.f, __builtin_inff());   // no value scales here: the reference follows the scores alone
  const _Float16* kb = a.k_buf + (int64_t)unit * a.buf_cap * kD;
  const _Float16* vb = a.v_buf + (int64_t)unit * a.buf_cap * kD;
  const int tau = lane & 31, cc = lane >> 5;   // value rows: this lane's token of the block, channel half

  // One block = 32 tokens: keys as the A operand (lane = token rho of tile t, channels 32s + 8g ..),
  // values as whole rows that go through the LDS transpose.  Rows past the end are clamped here and
  // masked by the causal test below.
  auto load_block = [&](int blk, u32x4 (&k)[2][4], u32x4 (&v)[8]) {
    const int t0 = 32 * blk;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int tok = min(t0 + 16 * t + rho, nb - 1);
#pragma unroll
      for (int s = 0; s < 4; ++s) k[t][s] = ldg128(kb + (int64_t)tok * kD + 32 * s + 8 * g);
    }
    const int tok = min(t0 + tau, nb - 1);
#pragma unroll
    for (int it = 0; it < 8; ++it) v[it] = ldg128(vb + (int64_t)tok * kD + 8 * (2 * it + cc));
  };

  u32x4 ka[2][4], va[8];   // the block being computed; the next one is in flight meanwhile
  if (blk0 < blk1) load_block(blk0, ka, va);
  for (int blk = blk0; blk < blk1; ++blk) {
    const int t0 = 32 * blk;
    u32x4 kn[2][4] = {}, vn[8] = {};
    if (blk + 1 < blk1) load_block(blk + 1, kn, vn);
    float x[NRT][8];   // raw scores, then exponents, then probabilities of this lane's eight tokens
    bool high = false;
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(ka[t][s]), qb[rt][s], acc, 0, 0, 0);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int tok = t0 + 16 * t + 4 * g + jj;
          x[rt][4 * t + jj] = tok < vis[rt] ? acc[jj] : -__builtin_inff();
        }
      }
      if (blk == blk0) {
        float s[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) s[j] = x[rt][j] * a.c0;
        first_reference(st, rt, s);
      }
      // masked tokens follow the visible ones, so a row either has its reference by now or sees nothing here
      const float shift = -st.m[rt];
      float top = -__builtin_inff();
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        x[rt][j] = __builtin_fmaf(x[rt][j], a.c0, shift);
        top = fmaxf(top, x[rt][j]);
      }
      high |= top > kTau;
    }
    if (__any(high)) {
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) raise_reference<false>(st, rt, x[rt]);
    }
    half8 pb[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float p = __builtin_amdgcn_exp2f(x[rt][j]);
        sum += p;
        pb[rt][j] = (_Float16)(p * kBufP);
      }
      st.l[rt] += sum;
    }

    wave_lds_sync();   // the previous block's LDS reads are done
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int ch = 8 * (2 * it + cc);
      const half8 v = as_half8(va[it]);
#pragma unroll
      for (int i = 0; i < 8; ++i) vt[ch + i][tau] = v[i];
    }
    wave_lds_sync();
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const _Float16* rowp = &vt[8 * rho + n][0];
      const uint2 lo = *reinterpret_cast<const uint2*>(rowp + 4 * g);
      const uint2 hi = *reinterpret_cast<const uint2*>(rowp + 16 + 4 * g);
      const half8 vop = as_half8((u32x4){lo.x, lo.y, hi.x, hi.y});
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt)
        st.o[rt][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vop, pb[rt], st.o[rt][n], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < 4; ++s) ka[t][s] = kn[t][s];
#pragma unroll
    for (int it = 0; it < 8; ++it) va[it] = vn[it];
  }
  write_partial<NRT, 16>(a, st, b, kvh, row0, split, 1.0f / kBufP);
}

// A wave carries NRT tiles of query rows: 16 in each but the last, TAIL (16 or 8) in the last.
// The kernels with one tile of at most 8 rows keep within 256 registers, so that two of their waves fit a SIMD;
// how many the planner asks for (one, mostly) is a measured choice, see make_plan.
template <int NRT, int TAIL, bool VERIFY, bool SINGLE, bool PAGED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(NRT == 1 && TAIL != 16 ? 2 : 1))) void attn_kernel(AttnArgs a) {
  __shared__ _Float16 vt[kD][kVtStride];   // value-tile transpose of the buffer chunk
  // Dispatch order: unit fastest, every quantized chunk before any buffer chunk.  The planner makes
  // no more quantized chunks than there are resident wave slots, so all of them start at once; the
  // short buffer chunks take the slots of the first waves to finish and end long before the last
  // quantized chunk does.  (Buffer chunks first cost the last 128 quantized chunks a 10 us late start.)
  const int unit = blockIdx.x, row0 = blockIdx.z * (16 * (NRT - 1) + TAIL);
  const int split = blockIdx.y;
  const int b = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  if (split < a.n_split_q)
    quant_chunk<NRT, TAIL, VERIFY, SINGLE, PAGED>(a, unit, b, kvh, row0, split);
  else
    buffer_chunk<NRT>(a, unit, b, kvh, row0, split, vt);
}

// One workgroup per compute unit: eight waves (two per SIMD) share 1/W of a unit's quantized groups
// (W = gridDim.y) and draw them one at a time from a counter in LDS, so a wave that the hardware
// serves faster - the older of the two waves of a SIMD wins every issue conflict, and finishes a
// fixed share tens of microseconds before the younger one - simply takes more groups, and the eight
// finish together.  Buffer chunks w, w + W, ... of the unit are the first items of the same queue.
// Each wave still writes one partial for its quantized groups (slot 8*w + wave).  For the draft calls
// that run faster with two waves per SIMD than with one: 2 - 8 query rows per kv-head, and one row
// (SINGLE) over a paged cache (see the planner); the planner guarantees at most four buffer items per
// workgroup (one transpose tile each).
template <bool SINGLE, bool PAGED>
__global__ __launch_bounds__(64 * kCuWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_kernel_cu(AttnArgs a) {
  __shared__ _Float16 vt[kCuBufItems][kD][kVtStride];
  __shared__ int queue;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int unit = blockIdx.x, w = blockIdx.y, n_wg = gridDim.y;
  const int b = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int n_groups = a.len.n_quant[b] / kG;
  const int g0 = (int)((int64_t)w * n_groups / n_wg), g1 = (int)((int64_t)(w + 1) * n_groups / n_wg);
  const int n_buf_items = w < a.n_split_b ? (a.n_split_b - w + n_wg - 1) / n_wg : 0;
  if (threadIdx.x == 0) queue = -n_buf_items;
  __syncthreads();
  auto draw = [&]() -> int {
    int v = 0;
    if (lane == 0) v = atomicAdd(&queue, 1);
    return __builtin_amdgcn_readfirstlane(v);
  };
  int c = draw();
  while (c < 0) {   // a buffer item: a partial of its own
    const int item = -c - 1;
    buffer_chunk<1>(a, unit, b, kvh, 0, a.n_split_q + w + n_wg * item, vt[item]);
    c = draw();
  }
  quant_chunk<1, 8, false, SINGLE, PAGED, true>(a, unit, b, kvh, 0, kCuWaves * w + wave, &queue, g0, g1 - g0, c);
}

// Merge of the per-chunk partials (Appendix E): M = max m_i, L = sum l_i 2^(m_i - M),
// out = sum o_i 2^(m_i - M) / L.  One 256-thread workgroup per query row: thread (sl, c) folds chunks
// sl, sl+8, ... for channels 4c..4c+3 into a running (m, l, o) of its own, nine chunks per step
// with all their loads issued together, so a row of up to 72 chunks (64 quantized + a decode-time
// buffer's) is one memory round trip; the eight slices are then combined through LDS.
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs a) {
  __shared__ float red_o[8][kD + 4];
  __shared__ float red_m[8], red_l[8];
  constexpr int U = 9;
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x, sl = tid >> 5, c = tid & 31;
  const float* __restrict__ ml = a.ws_ml + row * a.n_split * 2;
  const float* __restrict__ po = a.ws_o + row * a.n_split * kD + 4 * c;
  float m = kNegBig, l = 0.f;
  float4v o = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = sl; s0 < a.n_split; s0 += 8 * U) {
    float ms[U], ls[U];
    float4v xs[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = s0 + 8 * u;
      const int sc = min(s, a.n_split - 1);   // past the end: a valid address, weight 0
      const float2 p = *reinterpret_cast<const float2*>(ml + 2 * sc);
      ms[u] = s < a.n_split ? p.x : kNegBig;
      ls[u] = p.y;
      xs[u] = *reinterpret_cast<const float4v*>(po + (int64_t)sc * kD);
    }
    float mb = m;
#pragma unroll
    for (int u = 0; u < U; ++u) mb = fmaxf(mb, ms[u]);
    const float down = __builtin_amdgcn_exp2f(m - mb);
    l *= down;
    o *= down;
    m = mb;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float w = __builtin_amdgcn_exp2f(ms[u] - m);   // 0 for an empty chunk or past the end
      l = __builtin_fmaf(w, ls[u], l);
      o += w * xs[u];
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) red_o[sl][4 * c + i] = o[i];
  if (c == 0) {
    red_m[sl] = m;
    red_l[sl] = l;
  }
  __syncthreads();
  if (tid < kD) {
    float mm = red_m[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) mm = fmaxf(mm, red_m[k]);
    float os = 0.f, lsum = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float w = __builtin_amdgcn_exp2f(red_m[k] - mm);
      os = __builtin_fmaf(w, red_o[k][tid], os);
      lsum = __builtin_fmaf(w, red_l[k], lsum);
    }
    a.out[row * kD + tid] = (_Float16)(os / lsum);
    if (a.lse != nullptr && tid == 0) a.lse[row] = (mm + __builtin_log2f(lsum)) * 0.6931471805599453f;
  }
}

// ------------------------------------------------------------------------------------------------
// Other shapes than head_dim = group = 128 (plain layout, see quantspec.h).  One wave per workgroup, NRT
// tiles of 16 query rows, chunks are ranges of 32-token blocks.  The arithmetic is that of the kernels above:
//  * the codes lie in memory in the order the lanes of a wave take them as matrix-core operands: a
//    32-bit word holds the eight codes of one lane for one key step (eight channels of a token) or
//    one value tile (eight tokens of a channel).  A code c (4 or 8 bits), zero-extended to 16 bits,
//    is the fp16 subnormal c * 2^-24 and serves as the A operand of both contractions, exactly;
//  * keys: score = sum_c q_c (mul_c code_c + add_c) with (mul, add) = (S, Z) for the upper plane alone and
//    (S/16, Z - S/2) for the 8-bit code 16 C_U + C_L + 8.  Once per group of G tokens the row's queries and
//    the group's scales, each brought into a fixed range by a power of two, are multiplied in packed fp16
//    arithmetic: the rounded product and its exact remainder are the two operands hi + lo, and
//    sum_c q_c add_c becomes a per-row bias;
//  * values: out_c = sum_t (p_t mul_t) code_tc + sum_t p_t add_t per value group of the channel: the P operand
//    carries the value scale (and a power of two that follows the largest scale seen, so that it stays
//    inside fp16), the second sum is kept in binary32 beside the accumulators;
//  * the softmax reference of a row moves rarely (see the kernels above): a block's main path has no
//    cross-lane step;
//  * the full-precision buffer is the same block step with the fp16 rows as "codes" (keys straight from
//    memory, values transposed through LDS), q itself as the operand and no scales.
// Everything a block needs - its words, its value scales and zeros, the key scales and zeros of a group it
// starts - is requested one step before the block is worked on, through buffer resources, so that every
// step issues the same loads; the metadata passes through LDS from the lanes that loaded it to the lanes
// that use it.
// ------------------------------------------------------------------------------------------------
using half4 = _Float16 __attribute__((ext_vector_type(4)));

// Row `row` (of the n_rows that share kv-head kvh of sequence b) in the [B][nq][Hq] order of q and out.
__device__ __forceinline__ int64_t global_row(const AttnArgs& a, int b, int kvh, int row) {
  const int qi = row / a.rep, head = kvh * a.rep + row % a.rep;
  return ((int64_t)b * a.nq + qi) * a.n_q_heads + head;
}


// The eight codes of a word (C_U, or 16*C_U + C_L + 8 from the words of both planes) as 16-bit numbers: the
// matrix-core operand of the lane, element i = code i of the word.  Of the upper plane alone, elements 2, 3, 6
// and 7 come out 16 times too large (kLoneScale): the other operand makes up for it.
template <bool VERIFY>
__device__ __forceinline__ half8 code_operand(uint32_t u, uint32_t lw) {
  return VERIFY ? unpack8(u, lw) : unpack4(u);
}
constexpr float kLoneScale = 16.0f;
__host__ __device__ constexpr bool scaled_element(int i) { return (i & 2) != 0; }

// ONE: a single query row per kv-head (multi-head attention, one decode query): the quantized region takes the
// one-token-per-lane softmax of the kernels above.
template <int D, int G, bool VERIFY, int NRT, bool ONE = false>
__global__ __launch_bounds__(64, D == 256 ? (ONE ? 2 : 1) : (D == 64 && NRT == 1) ? 4 : 2) void attn_plain_kernel(AttnArgs a) {
  static_assert(!ONE || (NRT == 1 && !VERIFY), "the single-row path serves the draft call's one row");
  constexpr int KS = D / 32, NT = D / 16, VG = D / G;
  constexpr int PL = VERIFY ? 2 : 1;                  // planes read
  constexpr int VSTRIDE = 36;                         // 16-bit elements per LDS row (keeps 8-byte reads aligned)
  constexpr int kEvFloor = -40;                       // below every value scale that is not zero (2^-24 / 16)
  constexpr int kTauPlain = 6;                        // a score may exceed its row's reference by 2^6 before the reference is raised
  // LDS of the one wave: the two operands hi, lo of every (row tile, key step) for the quantized region, one
  // 16-byte slot per lane (a lane reads back what it wrote itself); or the values of a buffer block, [channel][token]
  // then (one tile of rows only: two would not leave room for eight waves per compute unit at head_dim 128) the
  // scaled queries in the same arrangement, and 4 D bytes through which a group's key scales and zeros pass
  // from the lanes that loaded them to the lanes that use them
  // (ONE: all 16 columns of the tile carry the one row, so the four lanes of a column share a slot with the
  // same lanes of every other column - a sixteenth of the room, which is what lets head_dim 256 run two waves per SIMD)
  constexpr bool kQInLds = NRT == 1;
  constexpr int QL = ONE ? 4 : 64;                    // operand slots per (part, tile, key step)
  constexpr int kOpBytes = 2 * NRT * KS * QL * 16, kQnBytes = kQInLds ? NRT * KS * QL * 16 : 0;
  constexpr int kVmBytes = 128 * VG;   // a block's value scales and zeros, likewise
  constexpr int kQBytes = kOpBytes + kQnBytes + 4 * D + kVmBytes, kVtBytes = D * VSTRIDE * 2;
  __shared__ __attribute__((aligned(16))) uint8_t lds[kQBytes > kVtBytes ? kQBytes : kVtBytes];
  uint8_t* const km_lds = lds + kOpBytes + kQnBytes;
  uint8_t* const vm_lds = km_lds + 4 * D;
  uint16_t (*vt)[VSTRIDE] = reinterpret_cast<uint16_t (*)[VSTRIDE]>(lds);
  const ShapeLayout lay{D, G};
  const int lane = threadIdx.x & 63, rho = lane & 15, g = lane >> 4;
  half8* q_lds = reinterpret_cast<half8*>(lds) + (ONE ? g : lane);   // operand (part, rt, s) at [((part * NRT + rt) * KS + s) * QL]
  half8* qn_lds = reinterpret_cast<half8*>(lds + kOpBytes) + (ONE ? g : lane);   // scaled queries (rt, s) at [(rt * KS + s) * QL]
  const int unit = blockIdx.x, split = blockIdx.y, row0 = blockIdx.z * 16 * NRT;
  const int b = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int nb = a.len.n_buf[b];
  const bool quantized = split < a.n_split_q;
  // this wave's range of 32-token blocks, of the quantized region or of the buffer
  const int n_blk = quantized ? a.len.n_quant[b] / 32 : (nb + 31) >> 5;
  const int piece = quantized ? split : split - a.n_split_q, pieces = quantized ? a.n_split_q : a.n_split_b;
  const int blk0 = (int)((int64_t)piece * n_blk / pieces), blk1 = (int)((int64_t)(piece + 1) * n_blk / pieces);

  const _Float16* qp[NRT];
  bool valid[NRT];
  int vis[NRT];   // buffer tokens [0, vis) are visible to this lane's query (causal among the nq queries)
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int row = ONE ? 0 : row0 + 16 * rt + rho;
    valid[rt] = row < a.n_rows;
    const int rowc = valid[rt] ? row : 0;
    const int qi = rowc / a.rep, head = kvh * a.rep + rowc % a.rep;
    qp[rt] = a.q + (((int64_t)b * a.nq + qi) * a.n_q_heads + head) * D + 8 * g;
    vis[rt] = valid[rt] ? nb - a.nq + qi + 1 : 0;
  }
  // operands of the query rows: q itself for the buffer (registers), hi and lo for the current group of keys (LDS)
  half8 qhi[NRT][KS];
  float sc[NRT], bias[NRT];
  auto load_q = [&](int rt, int s) {
    u32x4 w = ldg128(qp[rt] + 32 * s);
    if (!valid[rt]) w = (u32x4){0u, 0u, 0u, 0u};
    return as_half8(w);
  };
  auto plain_q = [&]() {
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
#pragma unroll
      for (int s = 0; s < KS; ++s) qhi[rt][s] = load_q(rt, s);
      sc[rt] = a.c0, bias[rt] = 0.f;
    }
  };
  // A row's queries are brought to |q| < 2^7 by a power of two, 2^fq (exact in fp16; at most 2^15, which only
  // leaves a row of tiny queries with less headroom than it could have)
  int fq[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    uint32_t qm = 0u;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 w = as_u32x4(load_q(rt, s));
#pragma unroll
      for (int r = 0; r < 4; ++r) qm = max_bits(qm, w[r] & 0x7FFF7FFFu);
    }
    const float qmax = group_max(larger_half(qm));
    fq[rt] = min(6 - max(exponent_of(qmax), -24), 15);
    if constexpr (kQInLds) {
      if (quantized) {
        const _Float16 up_q = (_Float16)pow2(fq[rt]);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const half8 qn = load_q(rt, s) * up_q;
          if (!ONE || rho == 0) qn_lds[(rt * KS + s) * QL] = qn;   // ONE: the columns hold the same; one of them writes
        }
      }
    }
  }
  // The operands of one group of keys.  The key scales are brought below 2^7 the same way (2^fs, from the
  // largest scale of the group over all channels), so a product q*S of the scaled numbers is below 2^14 and
  // splits into hi = fp16(q*S) and lo = q*S - hi without loss down to 2^-24: both are packed fp16 operations
  // (the remainder of an fp16 product is an fp16 number unless it underflows).
  // km: this lane's 16 bytes of the group's scales (lanes below D/8) and zeros (the D/8 lanes after them), as
  // they came with the block's words.  They go through LDS to the lanes that need them.
  auto scaled_q = [&](const u32x4& km) __attribute__((always_inline)) {
    wave_lds_sync();   // whoever still reads the previous group's numbers is done
    if (D == 256 || lane < D / 4) *reinterpret_cast<u32x4*>(km_lds + 16 * lane) = km;
    wave_lds_sync();
    u32x4 sw[KS], zw[KS];
    uint32_t sm = 0u;
    u32x4 qw[NRT][KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      sw[s] = *reinterpret_cast<const u32x4*>(km_lds + (32 * s + 8 * g) * 2);
      zw[s] = *reinterpret_cast<const u32x4*>(km_lds + 2 * D + (32 * s + 8 * g) * 2);
    }
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        if constexpr (kQInLds)
          qw[rt][s] = as_u32x4(qn_lds[(rt * KS + s) * QL]);
        else
          qw[rt][s] = as_u32x4(load_q(rt, s));   // everything is requested before anything is waited for
      }
    if constexpr (!kQInLds) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int r = 0; r < 4; ++r) sm = max_bits(sm, sw[s][r]);
    // the lanes of a row of 16 hold the same channels: the maximum over the four rows covers the group
    const float smax = group_max(larger_half(sm));
    const int fs = min(6 - max(exponent_of(smax), -24), 15);
    // the upper plane alone: the scale of an element whose code comes out 16 times too large is a sixteenth
    const _Float16 up_s = (_Float16)pow2(fs), up_s16 = (_Float16)pow2(fs - (VERIFY ? 0 : 4));
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      const _Float16 up_q = (_Float16)(kQInLds ? 1.0f : pow2(fq[rt]));
      float bz = 0.f, bs = 0.f;   // sum of q Z and of q S over this lane's channels, q scaled
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        u32x4 h4, l4;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const half2v qn = as_half2(qw[rt][s][r]) * up_q, sh = as_half2(sw[s][r]), zh = as_half2(zw[s][r]);
          const half2v sn = sh * (scaled_element(2 * r) ? up_s16 : up_s);
          const half2v hi = qn * sn;
          const half2v lo = __builtin_elementwise_fma(qn, sn, -hi);
          h4[r] = as_u32(hi), l4[r] = as_u32(lo);
          bz = __builtin_fmaf((float)qn[0], (float)zh[0], bz);
          bz = __builtin_fmaf((float)qn[1], (float)zh[1], bz);
          if (VERIFY) {
            bs = __builtin_fmaf((float)qn[0], (float)sh[0], bs);
            bs = __builtin_fmaf((float)qn[1], (float)sh[1], bs);
          }
        }
        if (!ONE || rho == 0) {
          q_lds[((0 * NRT + rt) * KS + s) * QL] = as_half8(h4);
          q_lds[((1 * NRT + rt) * KS + s) * QL] = as_half8(l4);
        }
      }
      // (mul, add) = (S, Z), or (S/16, Z - S/2) for both planes; 2^24 for a code read as a subnormal
      sc[rt] = a.c0 * pow2(24 - fq[rt] - fs - (VERIFY ? 4 : 0));
      bias[rt] = a.c0 * pow2(-fq[rt]) * group_sum(VERIFY ? __builtin_fmaf(-0.5f, bs, bz) : bz);
    }
  };

  float m[NRT], l[NRT], zs[NRT][VG];
  float4v o[NRT][NT];   // O^T accumulators: tile n, element jj -> channel 16*n + 4*g + jj
  int ev = quantized ? kEvFloor : 0;   // the P operand is p * mul * 2^(14 - kTauPlain - ev)
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    m[rt] = kNegBig, l[rt] = 0.f;
#pragma unroll
    for (int k = 0; k < VG; ++k) zs[rt][k] = 0.f;
#pragma unroll
    for (int n = 0; n < NT; ++n) o[rt][n] = (float4v){0.f, 0.f, 0.f, 0.f};
  }

  // ---- a block of the quantized region as it comes from memory ----
  struct Raw {
    uint32_t k[PL][2][KS];      // key words of the two 16-token tiles
    uint32_t v[PL][NT];         // value words
    u32x4 vm;                   // 16 bytes of the block's value scales (lanes below 4 VG) and zeros (the 4 VG lanes after them)
    u32x4 km;                   // 16 bytes of the key scales and zeros of the block's group, if the block starts one for the wave
  };
  // A block's words are requested one step before the block is worked on.  (Two steps, with a third set of
  // registers, changed no shape's time by more than 2 %: a wave's step is as long as its own instructions.)
  // Paged caches: where the 128-token row of the block to request in this step lies, and that of the step after
  // (the same in every lane): a table entry is asked for two steps before the block's words are, and waited for
  // there.  (The loop exists twice, with and without a table: table entries carried from step to step would
  // cost the cache without one a wait for every load in flight at the end of each step.)
  int place_load = 0, place_then = 0;
  auto logical_row = [&](int blk) -> int { return unit * (a.q_cap / kG) + (32 * min(blk, blk1 - 1)) / kSuper; };
  auto look_up = [&](int blk) -> int { return a.group_table[logical_row(blk)]; };
  // The words of block blk, requested through buffer resources that span the block's 128-token row: a block
  // that does not exist (exists == false: the one after the range's last) gets resources of no bytes, whose loads
  // return zero without touching memory - so every step of the loop issues the same loads and the waits
  // for a block's words can be counted, not drained.
  auto load_raw = [&](int blk, Raw& r, int place, bool exists) __attribute__((always_inline)) {
    const int64_t pg = place;
    const int st0 = (32 * blk) % kSuper;
    const __amdgpu_buffer_rsrc_t ru = block_resource(a.upper + pg * lay.upper_bytes(), exists ? lay.upper_bytes() : 0);
    {   // first, so that it is there first: lane l takes bytes [16 l, 16 l + 16) of the group's scales, then of its zeros
      const bool starts = exists && (blk == blk0 || st0 % G == 0);
      const __amdgpu_buffer_rsrc_t rm = block_resource(a.upper + pg * lay.upper_bytes(), starts ? lay.upper_bytes() : 0);
      const int half_lanes = D / 8, which = lane / half_lanes, piece16 = lane % half_lanes;
      const int off = (which == 0 ? lay.off_ks() : lay.off_kz()) + (st0 / G) * D * 2 + 16 * piece16;
      r.km = ldb128(rm, which < 2 ? off : lay.upper_bytes());
      const int whichv = lane / (4 * VG), piecev = lane % (4 * VG);
      const int offv = (whichv == 0 ? lay.off_vs() : lay.off_vz()) + st0 * VG * 2 + 16 * piecev;
      r.vm = ldb128(ru, whichv < 2 ? offv : lay.upper_bytes());
    }
    __amdgpu_buffer_rsrc_t rl = ru;
    if constexpr (PL == 2) rl = block_resource(a.lower + pg * lay.lower_bytes(), exists ? lay.lower_bytes() : 0);
#pragma unroll
    for (int pl = 0; pl < PL; ++pl) {
      const __amdgpu_buffer_rsrc_t rs = pl == 0 ? ru : rl;
      const int kp = lay.off_k(st0 / 32), vp = lay.off_v(st0 / 32);
      if constexpr (KS == 2) {   // head_dim 64: a lane's four words are the two key steps of both token tiles
        const u32x4 w = ldb128_stream(rs, kp + lane * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) r.k[pl][i >> 1][i & 1] = w[i];
      } else {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int sq = 0; sq < KS / 4; ++sq) {
            const u32x4 w = ldb128_stream(rs, kp + ((t * (KS / 4) + sq) * 64 + lane) * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) r.k[pl][t][4 * sq + i] = w[i];
          }
      }
#pragma unroll
      for (int nq = 0; nq < NT / 4; ++nq) {
        const u32x4 w = ldb128_stream(rs, vp + (nq * 64 + lane) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[pl][4 * nq + i] = w[i];
      }
    }
  };

  const uint16_t* kb = reinterpret_cast<const uint16_t*>(a.k_buf) + (int64_t)unit * a.buf_cap * D;
  const uint16_t* vb = reinterpret_cast<const uint16_t*>(a.v_buf) + (int64_t)unit * a.buf_cap * D;
  const int vtok = lane & 31, vhalf = lane >> 5;   // buffer values: lane (token, half) takes D/2 channels of one token
  auto fill_values = [&](int blk) {   // rows past the end are clamped here and masked below
    const int tok = min(32 * blk + vtok, nb - 1);
#pragma unroll
    for (int k = 0; k < D / 16; ++k) {
      const int ch0 = vhalf * (D / 2) + 8 * k;
      const u32x4 x = ldg128(vb + (int64_t)tok * D + ch0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vt[ch0 + 2 * e][vtok] = (uint16_t)(x[e] & 0xFFFFu);
        vt[ch0 + 2 * e + 1][vtok] = (uint16_t)(x[e] >> 16);
      }
    }
  };

  // one 32-token block; QUANT (a std::bool_constant): of the quantized region (its words in cur, those of the
  // next block requested into nxt), else of the buffer
  auto block_step = [&](int blk, auto QUANT, auto PAGED, Raw& cur, Raw& nxt) __attribute__((always_inline)) {
    constexpr bool quantized = decltype(QUANT)::value, paged = decltype(PAGED)::value;
    const int st0 = (32 * blk) % kSuper;   // first token of the block inside its 128-token row of the layout
    if constexpr (quantized) {
      if (blk == blk0 || st0 % G == 0) scaled_q(cur.km);   // the query operands of a new key group
      wave_lds_sync();   // the previous block's reads of these numbers are done
      if (VG == 8 || lane < 8 * VG) *reinterpret_cast<u32x4*>(vm_lds + 16 * lane) = cur.vm;
      load_raw(blk + 1, nxt, paged ? __builtin_amdgcn_readfirstlane(place_load) : logical_row(blk + 1), blk + 1 < blk1);
    } else {
      wave_lds_sync();   // the previous block's LDS reads are done
      fill_values(blk);
      wave_lds_sync();
    }
    // ---- scores, in log2 units ----
    float x[NRT][8], mx[NRT];
    bool high = false;
    float4v acc[NRT][2];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) acc[rt][0] = acc[rt][1] = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      half8 ka[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if constexpr (quantized)
          ka[t] = code_operand<VERIFY>(cur.k[0][t][s], cur.k[PL - 1][t][s]);
        else
          ka[t] = as_half8(ldg128(kb + (int64_t)min(32 * blk + 16 * t + rho, nb - 1) * D + 32 * s + 8 * g));
      }
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        if constexpr (quantized) {
          const half8 bh = q_lds[((0 * NRT + rt) * KS + s) * QL], bl = q_lds[((1 * NRT + rt) * KS + s) * QL];
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t], bh, acc[rt][t], 0, 0, 0);
            acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t], bl, acc[rt][t], 0, 0, 0);
          }
        } else {
#pragma unroll
          for (int t = 0; t < 2; ++t) acc[rt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t], qhi[rt][s], acc[rt][t], 0, 0, 0);
        }
      }
    }
    if constexpr (ONE && quantized) {
      // ---- one query row (carried by every column of the tile): its 32 scores sit eight per lane in the four lanes
      // of a column.  Those of column 0 are dealt out to lanes (k, g), k = 0..7 (lanes 8..15 mirror them): lane (k, g)
      // takes token 16 (k >> 2) + 4 g + (k & 3), so a
      // lane does one exponential and one multiply per value group; the fp16 products go back in pairs, which
      // completes the P operand in lane (0, g), the only column whose result is kept.  l and the zero-point sums
      // stay per lane and are folded over the eight lanes when the partial is written. ----
      auto bits = [](float f) { return __builtin_bit_cast(uint32_t, f); };
      uint32_t w = bits(acc[0][0][0]);
      w = row_shr_keep<1>(w, bits(acc[0][0][1]));
      w = row_shr_keep<2>(w, bits(acc[0][0][2]));
      w = row_shr_keep<3>(w, bits(acc[0][0][3]));
      w = row_shr_keep<4>(w, bits(acc[0][1][0]));
      w = row_shr_keep<5>(w, bits(acc[0][1][1]));
      w = row_shr_keep<6>(w, bits(acc[0][1][2]));
      w = row_shr_keep<7>(w, bits(acc[0][1][3]));
      w = (uint32_t)__builtin_amdgcn_update_dpp((int)w, (int)w, 0x118, 0xF, 0xC, false);   // lanes 8..15 <- lanes 0..7
      const float xv = __builtin_fmaf(__builtin_bit_cast(float, w), sc[0], bias[0]);
      const int kk = rho & 7, tok = 16 * (kk >> 2) + 4 * g + (kk & 3);
      using HV = _Float16 __attribute__((ext_vector_type(VG)));
      wave_lds_sync();
      const HV sv = *reinterpret_cast<const HV*>(vm_lds + tok * VG * 2);
      const HV zv = *reinterpret_cast<const HV*>(vm_lds + 64 * VG + tok * VG * 2);
      _Float16 sh_max = sv[0];
#pragma unroll
      for (int k = 1; k < VG; ++k) sh_max = __builtin_elementwise_max(sh_max, sv[k]);
      const float smax = (float)sh_max;
      const bool high = xv > m[0] + kTauPlain || exponent_of(smax) > ev;
      if (__any(high)) {   // as in the general path below; m, ev are the same in every lane
        const int eb = max(exponent_of(group_max(octet_max(smax))), ev);
        const float alpha_e = pow2(max(ev - eb, -120));
        ev = eb;
        const float m_new = fmaxf(m[0], group_max(octet_max(xv)));
        const float alpha = __builtin_amdgcn_exp2f(m[0] - m_new);
        m[0] = m_new;
        l[0] *= alpha;
#pragma unroll
        for (int k = 0; k < VG; ++k) zs[0][k] *= alpha;
        const float both = alpha * alpha_e;
#pragma unroll
        for (int n = 0; n < NT; ++n) o[0][n] *= both;
      }
      const float p = __builtin_amdgcn_exp2f(xv - m[0]);
      l[0] += p;
      // elements 2, 3, 6, 7 of the operand meet codes that come out 16 times too large
      const float ps = p * (pow2(14 - kTauPlain - ev) * ((rho & 2) ? 1.0f / kLoneScale : 1.0f));
      constexpr int TILES = NT / VG;
#pragma unroll
      for (int k = 0; k < VG; ++k) {
        zs[0][k] = __builtin_fmaf(p, (float)zv[k], zs[0][k]);
        const _Float16 h = (_Float16)__builtin_fmaf(ps, (float)sv[k], 0.f);
        const uint32_t hb = __builtin_bit_cast(uint16_t, h);
        const uint32_t pair = hb | (row_shl_zero<1>(hb) << 16);
        const half8 pb = as_half8((u32x4){pair, row_shl_zero<2>(pair), row_shl_zero<4>(pair), row_shl_zero<6>(pair)});
#pragma unroll
        for (int i = 0; i < TILES; ++i) {
          const int n = k * TILES + i;
          o[0][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(code_operand<false>(cur.v[0][n], 0u), pb, o[0][n], 0, 0, 0);
        }
      }
    } else {
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int tok = 32 * blk + 16 * t + 4 * g + jj;
          x[rt][4 * t + jj] = (quantized || tok < vis[rt]) ? __builtin_fmaf(acc[rt][t][jj], sc[rt], bias[rt]) : -__builtin_inff();
        }
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {   // this lane's tokens only: the rows' references move rarely (see below)
      mx[rt] = max_of(x[rt]);
      high |= mx[rt] > m[rt] + kTauPlain;
    }
    // ---- largest value scale of the block ----
    float smax = 0.f;
    uint2 vs[2][VG], vz[2][VG];   // value scale / zero of this lane's tokens 16 t + 4 g .. + 3: four tokens x VG groups
    if constexpr (quantized) {
      wave_lds_sync();
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int c = 0; c < VG; ++c) {
          vs[t][c] = *reinterpret_cast<const uint2*>(vm_lds + ((16 * t + 4 * g) * VG + 4 * c) * 2);
          vz[t][c] = *reinterpret_cast<const uint2*>(vm_lds + 64 * VG + ((16 * t + 4 * g) * VG + 4 * c) * 2);
        }
      uint32_t sm = 0u;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int c = 0; c < VG; ++c) sm = max_bits(sm, max_bits(vs[t][c].x, vs[t][c].y));
      smax = larger_half(sm);   // of this lane's tokens; all lanes of a group of 16 share their tokens
      high |= exponent_of(smax) - (VERIFY ? 4 : 0) > ev;
    }
    // m is a reference, not the running maximum: it is raised, to the maximum so far, only when a score exceeds
    // it by more than kTauPlain, so a probability is at most 2^kTauPlain and most blocks neither look across
    // lanes nor touch what is accumulated; the same branch raises the scale exponent when a larger value scale
    // appears.  A wave's first block always comes here (m starts at -infinity for all practical purposes).
    if (__any(high)) {
      const int eb = max(exponent_of(group_max(smax)) - (VERIFY ? 4 : 0), ev);
      const float alpha_e = pow2(max(ev - eb, -120));
      ev = eb;
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        const float m_new = fmaxf(m[rt], group_max(mx[rt]));
        const float alpha = __builtin_amdgcn_exp2f(m[rt] - m_new);
        m[rt] = m_new;
        l[rt] *= alpha;
#pragma unroll
        for (int k = 0; k < VG; ++k) zs[rt][k] *= alpha;
        const float both = alpha * alpha_e;
#pragma unroll
        for (int n = 0; n < NT; ++n) o[rt][n] *= both;
      }
    }
    const float pscale = pow2(14 - kTauPlain - ev) * (quantized && VERIFY ? 0.0625f : 1.0f);
    float xs[NRT][8];   // the probabilities with the power of two of the P operand
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        x[rt][j] = __builtin_amdgcn_exp2f(x[rt][j] - m[rt]);
        sum += x[rt][j];
        xs[rt][j] = x[rt][j] * (quantized && !VERIFY && scaled_element(j) ? pscale * (1.0f / kLoneScale) : pscale);
      }
      l[rt] += sum;
    }
    // ---- O^T[channel, column] += V^T x p, value group by value group ----
#pragma unroll
    for (int k = 0; k < (quantized ? VG : 1); ++k) {
      half8 pb[NRT];
      if constexpr (quantized) {
        // (mul, add) of token j = 4 t + jj of this lane: element (jj * VG + k) of the four-token run; they enter as
        // fp16 numbers (mixed-precision multiply-adds), the products are formed in binary32
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int idx = jj * VG + k, j = 4 * t + jj;
            const half4 s4 = __builtin_bit_cast(half4, vs[t][idx / 4]), z4 = __builtin_bit_cast(half4, vz[t][idx / 4]);
            const _Float16 sh = s4[idx % 4], zh = z4[idx % 4];
            if (VERIFY) {
              const float vadd = __builtin_fmaf(-0.5f, (float)sh, (float)zh);
#pragma unroll
              for (int rt = 0; rt < NRT; ++rt) zs[rt][k] = __builtin_fmaf(x[rt][j], vadd, zs[rt][k]);
            } else {
#pragma unroll
              for (int rt = 0; rt < NRT; ++rt) zs[rt][k] = __builtin_fmaf(x[rt][j], (float)zh, zs[rt][k]);
            }
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) pb[rt][j] = (_Float16)__builtin_fmaf(xs[rt][j], (float)sh, 0.f);
          }
      } else {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
          for (int j = 0; j < 8; ++j) pb[rt][j] = (_Float16)xs[rt][j];
      }
      constexpr int TILES = NT / VG;   // value tiles per value group (all of them for the buffer)
#pragma unroll
      for (int i = 0; i < (quantized ? TILES : NT); ++i) {
        const int n = quantized ? k * TILES + i : i;
        half8 vop;
        if constexpr (quantized) {
          vop = code_operand<VERIFY>(cur.v[0][n], cur.v[PL - 1][n]);
        } else {
          const uint16_t* rowp = &vt[16 * n + rho][0];
          const uint2 lo = *reinterpret_cast<const uint2*>(rowp + 4 * g);
          const uint2 hi = *reinterpret_cast<const uint2*>(rowp + 16 + 4 * g);
          vop = as_half8((u32x4){lo.x, lo.y, hi.x, hi.y});
        }
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
          o[rt][n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vop, pb[rt], o[rt][n], 0, 0, 0);
      }
    }
    }
    if constexpr (quantized && paged) place_load = place_then, place_then = look_up(blk + 3);
  };
  Raw ra, rb;
  // The two sets of registers swap roles from block to block, so the loop body is two steps; both always run (a
  // block left over follows the loop), which keeps the number of loads in flight known at every wait.
  auto quantized_range = [&](auto PAGED) __attribute__((always_inline)) {
    constexpr bool paged = decltype(PAGED)::value;
    const std::true_type Q{};
    if (blk0 >= blk1) return;
    load_raw(blk0, ra, paged ? look_up(blk0) : logical_row(blk0), true);
    if constexpr (paged) place_load = look_up(blk0 + 1), place_then = look_up(blk0 + 2);
    int blk = blk0;
    for (; blk + 1 < blk1; blk += 2) {
      block_step(blk, Q, PAGED, ra, rb);
      block_step(blk + 1, Q, PAGED, rb, ra);
    }
    if (blk < blk1) block_step(blk, Q, PAGED, ra, rb);
  };
  if (quantized) {
    if (a.group_table != nullptr)
      quantized_range(std::true_type{});
    else
      quantized_range(std::false_type{});
  } else {
    plain_q();
    for (int blk = blk0; blk < blk1; ++blk) block_step(blk, std::false_type{}, std::false_type{}, ra, rb);
  }
  // ---- partial: (m, l) and the unnormalised output row ----
  const int n_split = a.n_split_q + a.n_split_b;
  const float back = quantized ? pow2(ev + 10 + kTauPlain) : pow2(kTauPlain - 14);   // 2^(ev + tau - 14), and 2^24 for codes read as subnormals
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const bool spread = ONE && quantized;   // the sums lie one token per lane: over the eight lanes first
    const float lsum = group_sum(spread ? octet_sum(l[rt]) : l[rt]);
    float zsum[VG];
#pragma unroll
    for (int k = 0; k < VG; ++k) zsum[k] = group_sum(spread ? octet_sum(zs[rt][k]) : zs[rt][k]);
    const int row = row0 + 16 * rt + rho;
    if (row < a.n_rows) {
      const int64_t r = global_row(a, b, kvh, row) * n_split + split;
      float* po = a.ws_o + r * D;
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        float4v y;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) y[jj] = __builtin_fmaf(o[rt][n][jj], back, zsum[(16 * n) / G]);
        *reinterpret_cast<float4v*>(po + 16 * n + 4 * g) = y;
      }
      if (g == 0) {
        a.ws_ml[2 * r] = m[rt];
        a.ws_ml[2 * r + 1] = lsum;
      }
    }
  }
}

// Merge for any head_dim: thread (sl, c) folds chunks sl, sl + SL, ... for channels 4c .. 4c+3; the SL
// slices are then combined through LDS (see merge_kernel).
template <int D>
__global__ __launch_bounds__(256) void merge_plain_kernel(MergeArgs a) {
  constexpr int CL = D / 4, SL = 256 / CL;
  __shared__ float red_o[SL][D + 4];
  __shared__ float red_m[SL], red_l[SL];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x, sl = tid / CL, c = tid % CL;
  const float* ml = a.ws_ml + row * a.n_split * 2;
  const float* po = a.ws_o + row * a.n_split * D + 4 * c;
  float m = kNegBig, l = 0.f;
  float4v o = {0.f, 0.f, 0.f, 0.f};
  for (int s = sl; s < a.n_split; s += SL) {
    const float2 p = *reinterpret_cast<const float2*>(ml + 2 * s);
    const float4v x = *reinterpret_cast<const float4v*>(po + (int64_t)s * D);
    const float mb = fmaxf(m, p.x);
    const float down = __builtin_amdgcn_exp2f(m - mb), w = __builtin_amdgcn_exp2f(p.x - mb);
    l = __builtin_fmaf(w, p.y, l * down);
    o = o * down + w * x;
    m = mb;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) red_o[sl][4 * c + i] = o[i];
  if (c == 0) red_m[sl] = m, red_l[sl] = l;
  __syncthreads();
  if (tid < D) {
    float mm = red_m[0];
#pragma unroll
    for (int k = 1; k < SL; ++k) mm = fmaxf(mm, red_m[k]);
    float os = 0.f, lsum = 0.f;
#pragma unroll
    for (int k = 0; k < SL; ++k) {
      const float w = __builtin_amdgcn_exp2f(red_m[k] - mm);
      os = __builtin_fmaf(w, red_o[k][tid], os);
      lsum = __builtin_fmaf(w, red_l[k], lsum);
    }
    a.out[row * D + tid] = (_Float16)(os / lsum);
    if (a.lse != nullptr && tid == 0) a.lse[row] = (mm + __builtin_log2f(lsum)) * 0.6931471805599453f;
  }
}

template <int D, int G>
hipError_t launch_attn_plain(const AttnArgs& a, int batch, bool verify, hipStream_t s) {
  // two row tiles per wave where their accumulators fit the register file (head_dim 256: 128 of them per tile)
  const int nrt = (D == 256 || a.n_rows <= 16) ? 1 : 2;
  dim3 grid(batch * a.n_kv_heads, a.n_split_q + a.n_split_b, (a.n_rows + 16 * nrt - 1) / (16 * nrt));
  if constexpr (D != 256) {
    if (nrt == 2)
      return verify ? launch(attn_plain_kernel<D, G, true, 2>, grid, dim3(64), s, a)
                    : launch(attn_plain_kernel<D, G, false, 2>, grid, dim3(64), s, a);
  }
  if (!verify && a.n_rows == 1) return launch(attn_plain_kernel<D, G, false, 1, true>, grid, dim3(64), s, a);
  return verify ? launch(attn_plain_kernel<D, G, true, 1>, grid, dim3(64), s, a)
                : launch(attn_plain_kernel<D, G, false, 1>, grid, dim3(64), s, a);
}

template <int NRT, int TAIL, bool VERIFY, bool SINGLE = false>
hipError_t launch_attn_kernel(const AttnArgs& a, dim3 grid, hipStream_t s) {
  return a.group_table != nullptr ? launch(attn_kernel<NRT, TAIL, VERIFY, SINGLE, true>, grid, dim3(64), s, a)
                                  : launch(attn_kernel<NRT, TAIL, VERIFY, SINGLE, false>, grid, dim3(64), s, a);
}

hipError_t launch_attn_cu(const AttnArgs& a, dim3 grid, hipStream_t s) {
  if (a.n_rows == 1) return launch(attn_kernel_cu<true, true>, grid, dim3(64 * kCuWaves), s, a);
  return a.group_table != nullptr ? launch(attn_kernel_cu<false, true>, grid, dim3(64 * kCuWaves), s, a)
                                  : launch(attn_kernel_cu<false, false>, grid, dim3(64 * kCuWaves), s, a);
}

template <int NRT, int TAIL>
hipError_t launch_attn_tiles(const AttnArgs& a, int batch, bool verify, hipStream_t s) {
  constexpr int rows = 16 * (NRT - 1) + TAIL;
  dim3 grid(batch * a.n_kv_heads, a.n_split_q + a.n_split_b, (a.n_rows + rows - 1) / rows);
  return verify ? launch_attn_kernel<NRT, TAIL, true>(a, grid, s) : launch_attn_kernel<NRT, TAIL, false>(a, grid, s);
}

}  // namespace

// Query rows per kv-head -> tiles of the wave: up to 8 rows one tile with the remainders in its other
// columns; up to 16 one full tile; up to 24 a full tile and one of 8; up to 32 two full tiles; more: row
// batches of 32 over grid.z.
hipError_t launch_attn(const AttnArgs& a, int batch, bool verify, hipStream_t s) {
  if (a.head_dim != kD || a.group != kG) {
#define QS_SHAPE(DD, GG) \
  if (a.head_dim == DD && a.group == GG) return launch_attn_plain<DD, GG>(a, batch, verify, s);
    QS_SHAPE(64, 32) QS_SHAPE(64, 64) QS_SHAPE(128, 32) QS_SHAPE(128, 64) QS_SHAPE(256, 32) QS_SHAPE(256, 64) QS_SHAPE(256, 128)
#undef QS_SHAPE
    return hipErrorInvalidValue;
  }
  if (a.cu_wgs > 0) {   // a draft call the planner wants two waves per SIMD for: one workgroup per compute unit, groups drawn dynamically
    if (verify || a.n_rows > 8 || (a.n_rows == 1 && a.group_table == nullptr)) return hipErrorInvalidValue;
    return launch_attn_cu(a, dim3(batch * a.n_kv_heads, a.cu_wgs, 1), s);
  }
  if (a.n_rows == 1 && !verify) {   // one query row per kv-head: one token per lane in the softmax
    dim3 grid(batch * a.n_kv_heads, a.n_split_q + a.n_split_b, 1);
    return launch_attn_kernel<1, 8, false, true>(a, grid, s);
  }
  if (a.n_rows <= 8) return launch_attn_tiles<1, 8>(a, batch, verify, s);
  if (a.n_rows <= 16) return launch_attn_tiles<1, 16>(a, batch, verify, s);
  if (a.n_rows <= 24) return launch_attn_tiles<2, 8>(a, batch, verify, s);
  return launch_attn_tiles<2, 16>(a, batch, verify, s);
}

hipError_t launch_merge(const MergeArgs& a, int rows_total, hipStream_t s) {
  if (a.head_dim == 64) return launch(merge_plain_kernel<64>, dim3(rows_total), dim3(256), s, a);
  if (a.head_dim == 256) return launch(merge_plain_kernel<256>, dim3(rows_total), dim3(256), s, a);
  return launch(merge_kernel, dim3(rows_total), dim3(256), s, a);
}

}  // namespace qs
