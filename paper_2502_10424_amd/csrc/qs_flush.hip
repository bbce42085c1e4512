// Quantize-on-flush, buffer move and plane export kernels (gfx950).
//
// Encoding (paper Section 4.2): per group, Z = min, S = (max - min)/15 stored as fp16; then with
// the stored S and Z, in binary32 and one rounding per operation (this file is compiled with
// -ffp-contract=off):  C_U = clamp(rne((x - Z)/S), 0, 15);  E_U = x - (C_U*S + Z);
// C_L = clamp(rne(E_U / (S/16)), -8, 7).  Keys are grouped per channel over 128 tokens, values per
// token over the 128 channels (Section 4.3.1).
//
// One workgroup of 256 threads handles one 128-token group of one (sequence, kv-head) unit, keys
// and values together.  Thread (c8 = tid & 15, oct = tid >> 4) owns channels [8*c8, 8*c8+8) of the
// eight tokens that share one 32-bit word of the value-plane tile, so every value word and every
// key word is assembled in registers and each plane is written exactly once.
#include "qs_internal.h"

namespace qs {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ half8 ld_half8(const _Float16* p) {
  return *reinterpret_cast<const half8*>(p);
}

// Token (inside a 32-token value tile) that sits at operand position j of lane group g, and the
// nibble of the 32-bit word that holds it.  The attention kernel consumes exactly this order.
__device__ __forceinline__ int tile_token(int g, int j) { return ((j >> 2) << 4) + 4 * g + (j & 3); }
__device__ __forceinline__ int tile_nibble(int j) { return ((j & 1) << 2) + (j >> 1); }

struct Codes {
  uint32_t u, l;   // C_U and C_L + 8, both in [0, 15]
};

__device__ __forceinline__ Codes encode(float x, float s, float z) {
  float t = (x - z) / s;
  float u = fminf(fmaxf(rintf(t), 0.0f), 15.0f);
  float deq = u * s;
  deq = deq + z;
  float e = x - deq;
  float sl = s / 16.0f;
  float l = fminf(fmaxf(rintf(e / sl), -8.0f), 7.0f);
  Codes c;
  c.u = (uint32_t)(int)u;
  c.l = (uint32_t)((int)l + 8);
  return c;
}

__device__ __forceinline__ _Float16 make_scale(float mn, float mx) {
  float s = (mx - mn) / 15.0f;
  _Float16 h = (_Float16)s;
  if (h == (_Float16)0.0f) h = (_Float16)1.0f;
  return h;
}

__global__ __launch_bounds__(256) void flush_kernel(FlushArgs a) {
  __shared__ float red[4][128][2];
  const int grp = blockIdx.x, unit = blockIdx.y;
  const int b = unit / a.n_kv_heads;
  const int tid = threadIdx.x, c8 = tid & 15, oct = tid >> 4, blk = oct >> 2, g = oct & 3;
  const int wave = tid >> 6;
  const int tq0 = a.n_quant[b] + grp * kG;     // destination token offset inside the unit
  const _Float16* ksrc = a.k_src + ((int64_t)unit * a.src_stride + (int64_t)grp * kG) * kD + 8 * c8;
  const _Float16* vsrc = a.v_src + ((int64_t)unit * a.src_stride + (int64_t)grp * kG) * kD + 8 * c8;

  half8 kx[8], vx[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int tok = 32 * blk + tile_token(g, j);
    kx[j] = ld_half8(ksrc + (int64_t)tok * kD);
    vx[j] = ld_half8(vsrc + (int64_t)tok * kD);
  }

  // ---- keys: min / max per channel over the 128 tokens of the group -------------------------
  float kmn[8], kmx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float mn = (float)kx[0][i], mx = mn;
#pragma unroll
    for (int j = 1; j < 8; ++j) {
      mn = fminf(mn, (float)kx[j][i]);
      mx = fmaxf(mx, (float)kx[j][i]);
    }
    // the four lane groups of a wave hold the other tokens of this 32-token tile
    mn = fminf(mn, __shfl_xor(mn, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mn = fminf(mn, __shfl_xor(mn, 32));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    kmn[i] = mn;
    kmx[i] = mx;
  }
  if (g == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      red[wave][8 * c8 + i][0] = kmn[i];
      red[wave][8 * c8 + i][1] = kmx[i];
    }
  }
  __syncthreads();
  float ks[8], kz[8];
  half8 ksh, kzh;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float mn = red[0][8 * c8 + i][0], mx = red[0][8 * c8 + i][1];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      mn = fminf(mn, red[w][8 * c8 + i][0]);
      mx = fmaxf(mx, red[w][8 * c8 + i][1]);
    }
    ksh[i] = make_scale(mn, mx);
    kzh[i] = (_Float16)mn;
    ks[i] = (float)ksh[i];
    kz[i] = mn;
  }
  const int64_t grp_dst = (int64_t)unit * (a.q_cap / kG) + tq0 / kG;
  if (oct == 0) {
    // stored in the order the attention kernel's B operand wants them: [k-step][lane group][element]
    half8 so, zo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      so[e] = ksh[tile_nibble(e)];
      zo[e] = kzh[tile_nibble(e)];
    }
    const int pos = (c8 & 3) * 32 + (c8 >> 2) * 8;
    *reinterpret_cast<half8*>(a.k_scale + grp_dst * kD + pos) = so;
    *reinterpret_cast<half8*>(a.k_zero + grp_dst * kD + pos) = zo;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint32_t wu = 0, wl = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      Codes c = encode((float)kx[j][i], ks[i], kz[i]);
      wu |= c.u << (4 * i);
      wl |= c.l << (4 * i);
    }
    const int tok = 32 * blk + tile_token(g, j);
    const int64_t w = ((int64_t)unit * a.q_cap + tq0 + tok) * kRowDw + c8;
    a.k_upper[w] = wu;
    a.k_lower[w] = wl;
  }

  // ---- values: min / max per token over its 128 channels --------------------------------------
  half8 vsh, vzh;
  uint32_t vu[8], vl[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) vu[i] = vl[i] = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float mn = (float)vx[j][0], mx = mn;
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      mn = fminf(mn, (float)vx[j][i]);
      mx = fmaxf(mx, (float)vx[j][i]);
    }
#pragma unroll
    for (int sft = 1; sft < 16; sft <<= 1) {   // the 16 lanes c8 = 0..15 hold the token's other channels
      mn = fminf(mn, __shfl_xor(mn, sft));
      mx = fmaxf(mx, __shfl_xor(mx, sft));
    }
    vsh[j] = make_scale(mn, mx);
    vzh[j] = (_Float16)mn;
    const float s = (float)vsh[j], z = mn;
    const int nib = 4 * tile_nibble(j);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      Codes c = encode((float)vx[j][i], s, z);
      vu[i] |= c.u << nib;
      vl[i] |= c.l << nib;
    }
  }
  const int64_t tile = (int64_t)unit * (a.q_cap / kVTileTok) + tq0 / kVTileTok + blk;
  if (c8 == 0) {
    const int64_t m = (int64_t)unit * a.q_cap + tq0 + 32 * blk + 8 * g;
    *reinterpret_cast<half8*>(a.v_scale + m) = vsh;
    *reinterpret_cast<half8*>(a.v_zero + m) = vzh;
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t w = tile * kVTileDw + (h * 64 + 16 * g + c8) * 4;
    *reinterpret_cast<uint4*>(a.v_upper + w) = make_uint4(vu[4 * h], vu[4 * h + 1], vu[4 * h + 2], vu[4 * h + 3]);
    *reinterpret_cast<uint4*>(a.v_lower + w) = make_uint4(vl[4 * h], vl[4 * h + 1], vl[4 * h + 2], vl[4 * h + 3]);
  }
}

// Buffer move (Section 4.3.2): rows [n_tokens, n_buf) become rows [0, n_buf - n_tokens).  Source and
// destination may overlap.  Thread (lane = tid >> 4, c = tid & 15) walks rows lane, lane+16, ...
// of its own 16-byte column; n_tokens is a multiple of 16, so the row a thread overwrites was read
// by the same thread in an earlier iteration and no cross-thread ordering is needed.
__global__ __launch_bounds__(256) void shift_kernel(ShiftArgs a) {
  const int unit = blockIdx.x;
  const int b = unit / a.n_kv_heads;
  _Float16* buf = (blockIdx.y == 0 ? a.k_buf : a.v_buf) + (int64_t)unit * a.buf_cap * kD;
  const int n_keep = a.n_buf[b] - a.n_tokens;
  const int c = threadIdx.x & 15;
  for (int r = threadIdx.x >> 4; r < n_keep; r += 16) {
    uint4 x = *reinterpret_cast<const uint4*>(buf + (int64_t)(r + a.n_tokens) * kD + 8 * c);
    *reinterpret_cast<uint4*>(buf + (int64_t)r * kD + 8 * c) = x;
  }
}

// Expand packed planes into one code per byte, plain [token][channel] order.
__global__ __launch_bounds__(256) void export_kernel(ExportArgs a) {
  const int idx = blockIdx.x * 256 + threadIdx.x;      // one 32-bit word of each plane
  if (idx >= a.n_tokens * kRowDw) return;
  {  // keys: word idx = token * 16 + c8
    const int tok = idx >> 4, c8 = idx & 15;
    const uint32_t wu = a.k_upper[idx], wl = a.k_lower[idx];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (a.k_u) a.k_u[tok * kD + 8 * c8 + i] = (uint8_t)((wu >> (4 * i)) & 15u);
      if (a.k_l) a.k_l[tok * kD + 8 * c8 + i] = (int8_t)((int)((wl >> (4 * i)) & 15u) - 8);
    }
  }
  {  // values: word idx = tile * 512 + (h*64 + 16*g + m)*4 + i
    const int tile = idx >> 9, w = idx & 511;
    const int h = w >> 8, g = (w >> 6) & 3, m = (w >> 2) & 15, i = w & 3;
    const int ch = 8 * m + 4 * h + i;
    const uint32_t wu = a.v_upper[idx], wl = a.v_lower[idx];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok = 32 * tile + tile_token(g, j);
      const int nib = 4 * tile_nibble(j);
      if (a.v_u) a.v_u[tok * kD + ch] = (uint8_t)((wu >> nib) & 15u);
      if (a.v_l) a.v_l[tok * kD + ch] = (int8_t)((int)((wl >> nib) & 15u) - 8);
    }
  }
  if (idx < a.n_tokens) {  // key metadata: position 32*s + 8*g + e of a group -> channel 32*g + 8*s + nibble(e)
    const int grp = idx >> 7, pos = idx & 127;
    const int ch = 32 * ((pos >> 3) & 3) + 8 * (pos >> 5) + tile_nibble(pos & 7);
    if (a.k_s) a.k_s[grp * kD + ch] = a.k_scale[idx];
    if (a.k_z) a.k_z[grp * kD + ch] = a.k_zero[idx];
  }
  if (idx < a.n_tokens) {  // value metadata: position 8*g + j of a tile -> token order
    const int tile = idx >> 5, p = idx & 31;
    const int tok = 32 * tile + tile_token(p >> 3, p & 7);
    if (a.v_s) a.v_s[tok] = a.v_scale[idx];
    if (a.v_z) a.v_z[tok] = a.v_zero[idx];
  }
}

}  // namespace

hipError_t launch_flush(const FlushArgs& a, int batch, hipStream_t s) {
  if (a.n_groups <= 0) return hipSuccess;
  dim3 grid(a.n_groups, batch * a.n_kv_heads);
  hipLaunchKernelGGL(flush_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_shift(const ShiftArgs& a, int batch, hipStream_t s) {
  dim3 grid(batch * a.n_kv_heads, 2);
  hipLaunchKernelGGL(shift_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_export(const ExportArgs& a, hipStream_t s) {
  if (a.n_tokens <= 0) return hipSuccess;
  const int words = a.n_tokens * kRowDw;
  hipLaunchKernelGGL(export_kernel, dim3((words + 255) / 256), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace qs
