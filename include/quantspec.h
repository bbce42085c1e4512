/*
 * quantspec.h - C ABI of the MI355X (gfx950) decode-attention library for QuantSpec's
 * hierarchical 4-bit KV cache.
 *
 * The three operations are the per-layer cache operations of the paper's Algorithm 1:
 *   qs_quantize_flush  - QUANTIZE(C_F1) appended to C_U, C_L, then the buffer move   (Section 4.3.2)
 *   qs_attn_draft      - attention of DRAFT : upper 4-bit plane C_U + full-precision buffer
 *   qs_attn_verify     - attention of TARGET: C_U and C_L (INT8 = 16 C_U + C_L) + buffer,
 *                        gamma + 1 query tokens, causal among them                     (Section 4.2)
 *
 * General rules
 *   - Every pointer inside qs_cache except n_quant / n_buf is a DEVICE pointer owned by the
 *     caller; n_quant and n_buf are HOST arrays read during the call (they are copied into the
 *     kernel arguments, so they may change as soon as the call returns).
 *   - The library never allocates, frees or synchronizes.  Every call enqueues its kernels on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *   - Return value: QS_OK, or a negative qs_status; on error nothing has been enqueued.  There is no
 *     process-wide state: what a call does depends on its arguments (and the current device) alone.
 *   - Shapes: head_dim D in {64, 128, 256} and group G in {32, 64, 128} with G dividing D (Section
 *     4.3.1 leaves both open).  D = G = 128, the paper's evaluation setting (Section 5.1), has its own
 *     layout and kernels, tuned to the memory roofline; the other shapes share a plain layout and one
 *     simpler, slower set of kernels with the same arithmetic and the same accuracy.  Wherever this header
 *     writes 128 for a channel count or a group of tokens in a signature, read D or G.
 *   - All device pointers must be 16-byte aligned.
 *
 * Cache layout (B = batch, Hkv = n_kv_heads, "unit" = one (sequence, kv-head) pair)
 *   The quantized region is two arrays, the paper's C_U and C_L, cut into blocks of 32 tokens so that
 *   the draft pass streams one array and the target pass two, each front to back:
 *     upper : uint8 [B][Hkv][q_cap/32][4352]   per block
 *               [   0, 2048)  key codes C_U, 32 token rows of 64 bytes: byte j of a row holds channel 2j
 *                             in bits 0-3 and channel 2j+1 in bits 4-7
 *               [2048, 4096)  value codes C_U, tiled for the matrix-core operand: 32-bit word
 *                             ((h*64 + 16*g + m)*4 + i) holds channel 8*m + 4*h + i (h<2, g<4, m<16, i<4)
 *                             of eight tokens; nibble (j&1)*4 + (j>>1) (j<8) belongs to token
 *                             (j>>2)*16 + 4*g + (j&3) of the block
 *               [4096, 4160)  value scale S, fp16, one per token, at position 8*g + j for the token above
 *               [4160, 4224)  value zero Z, same order
 *               [4224, 4288)  key scale S, fp16: 32 of the 128 per-channel values of the block's
 *                             128-token group.  Block p (= block index mod 4) of a group holds positions
 *                             [32p, 32p+32) of the group's operand order, in which position
 *                             32*s + 8*g + e (s<4, g<4, e<8) is channel 32*g + 8*s + (e&1)*4 + (e>>1)
 *               [4288, 4352)  key zero Z, same order
 *     lower : uint8 [B][Hkv][q_cap/32][4096]   per block
 *               [   0, 2048)  key codes C_L + 8 (0..15), same arrangement as in the upper array
 *               [2048, 4096)  value codes C_L + 8, likewise
 *   Other shapes (D, G) than (128, 128): both arrays are cut into rows of 128 tokens (four blocks of 32), VG = D/G
 *   value groups per token, 128/G key groups per row.  Codes are packed eight to a 32-bit word, one word per lane
 *   of a 64-lane wave (lane = 16*g + r, g < 4, r < 16) and matrix-core step; the word's code i (i < 8) sits in
 *   nibble (i&1)*4 + (i>>1), i.e. bits 4*nibble .. 4*nibble+3, as in the value words above:
 *     upper : uint8 [B][Hkv][q_cap/128][128*D + 1024*VG]   per row
 *               block p (p < 4) at 32*D*p:
 *                 [0, 16*D)           key codes C_U: word ((t*(D/128) + s/4)*64 + lane)*4 + s%4 (D = 64: word
 *                                     4*lane + 2*t + s) holds channels 32*s + 8*g + i of token 32*p + 16*t + r
 *                                     (t < 2, s < D/32)
 *                 [16*D, 32*D)        value codes C_U: word ((n/4)*64 + lane)*4 + n%4 (n < D/16) holds channel
 *                                     16*n + r of tokens 32*p + 16*(i/4) + 4*g + i%4
 *               [128*D, ...)          fp16, plain order: value scale S [128][VG], value zero Z [128][VG],
 *                                     key scale S [128/G][D], key zero Z [128/G][D]
 *     lower : uint8 [B][Hkv][q_cap/128][128*D]             per row: the codes C_L + 8, arranged as in upper
 *   Paging: by default unit u = b*Hkv + kv_head owns the q_cap/128 consecutive 128-token groups (four
 *   blocks, or one row of the other shapes' layout, each; the unit of paging whatever G is) that start at
 *   group u*(q_cap/128) of both arrays.  With a group table
 *   (group_table != NULL) entry [b][kv_head][g] is instead the index, counted in groups, of the place
 *   in upper / lower that holds logical group g of that unit: upper and lower are then pools of
 *   pool_groups groups in any order, and q_cap is only the longest a sequence may get.
 *   Keys are grouped per channel over G consecutive tokens, values per token over G consecutive channels
 *   (Section 4.3.1); both planes share S and Z.  qs_quantize_flush / qs_quantize_prefill are the only
 *   writers of these arrays; qs_export_codes returns plain [token][channel] codes and metadata.
 *   Full-precision buffer (Section 4.3.2), plain row-major, written by the caller or by qs_append:
 *     k_buf, v_buf     : fp16  [B][Hkv][buf_cap][D]     tokens [0, n_buf[b]) are valid.
 *   A cache may have no quantized region at all: q_cap == 0, n_quant[b] == 0, and upper / lower may
 *   then be NULL.  The attention calls are then plain fp16 attention over the
 *   buffer, of any length up to buf_cap (the full-precision baseline of the paper's Table 4).
 */
#ifndef QUANTSPEC_H_
#define QUANTSPEC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QS_MAX_BATCH 256    /* per-sequence lengths travel by value in the kernel arguments      */
#define QS_MAX_NQ 16        /* largest number of query tokens per sequence in one verify call    */
#define QS_STATIC_WS_BYTES (32u << 20)   /* device scratch built into the library, see qs_attn_static  */

/* qs_cache.flags.  Not part of the method: they select between equivalent ways of dealing the work of
 * Appendix E's chunked decode out to the chip.
 *   QS_FLAG_FIXED_RANGES  every wave of the attention kernels gets a fixed range of 128-token groups, so
 *                         results are bit-reproducible from call to call.  That is how most calls run
 *                         anyway; without the flag (default) qs_attn_draft at head_dim = group = 128 with
 *                         2 to 8 query heads per kv-head, or with one over a paged cache, lets the waves
 *                         of a compute unit draw their groups from a shared queue at run time: 3 - 9 %
 *                         faster at 128k context, but which partial sum a group lands in - and with it
 *                         the last bit of an fp16 output - can differ between calls.                    */
#define QS_FLAG_FIXED_RANGES 1u

typedef enum qs_status {
  QS_OK = 0,
  QS_ERR_NULL = -1,         /* a required pointer is NULL                                         */
  QS_ERR_SHAPE = -2,        /* batch / head counts / capacities are inconsistent                  */
  QS_ERR_UNSUPPORTED = -3,  /* (head_dim, group) not listed above, batch > QS_MAX_BATCH, nq > QS_MAX_NQ */
  QS_ERR_ALIGN = -4,        /* a device pointer is not 16-byte aligned                            */
  QS_ERR_RANGE = -5,        /* a length exceeds its capacity, is not a multiple of the group, n_buf < nq;
                               compute_units or flags out of range                                  */
  QS_ERR_WORKSPACE = -6,    /* workspace missing or smaller than qs_workspace_bytes()              */
  QS_ERR_HIP = -7           /* a HIP runtime call failed (no device, launch failure)               */
} qs_status;

typedef struct qs_cache {
  int32_t batch, n_q_heads, n_kv_heads;   /* n_q_heads % n_kv_heads == 0 (grouped-query attention)   */
  int32_t head_dim, group;                /* D and G, see "Shapes" above                              */
  int32_t q_cap;                          /* capacity of the quantized region in tokens, multiple of 128 */
  int32_t buf_cap;                        /* capacity of the fp16 buffer in tokens                    */
  void *upper, *lower;                    /* device, C_U and C_L, see layout above                    */
  void *k_buf, *v_buf;
  const int32_t *n_quant;                 /* HOST int32[batch]: valid quantized tokens (multiple of group) */
  const int32_t *n_buf;                   /* HOST int32[batch]: valid buffer tokens                   */
  const int32_t *group_table;             /* DEVICE int32 [batch][n_kv_heads][q_cap/128], or NULL = contiguous.
                                             Entries must lie in [0, pool_groups) and be distinct where the
                                             groups are live; the library cannot check device memory        */
  int32_t pool_groups;                    /* groups held by upper / lower when group_table is given        */
  int32_t compute_units;                  /* compute units the attention calls are planned for, e.g. when part
                                             of the GPU is reserved for other work; 0 = all of the current device's */
  uint32_t flags;                         /* QS_FLAG_*; 0 = defaults                                        */
} qs_cache;

/* Library version: major*10000 + minor*100 + patch. */
int qs_version(void);

/* Static, NUL-terminated description of a qs_status code. */
const char *qs_strerror(int code);

/*
 * Bytes of device scratch the attention calls need for their split-K partial results
 * (Appendix E: per-chunk partials that are merged afterwards).  Depends only on the descriptor
 * (shapes, capacities, compute_units, flags; with compute_units == 0 also on the current device) and
 * on nq (1 for draft), not on the current lengths, so it can be sized once.  Returns 0 if `c` is invalid.
 */
size_t qs_workspace_bytes(const qs_cache *c, int32_t nq);

/*
 * QUANTIZE on flush (Section 4.2, Section 4.3.2; the step of Algorithm 1's decode loop that quantizes
 * the older half of the full-precision buffer once it is full): for every sequence b, quantize buffer tokens [0, n_tokens) into both
 * 4-bit planes with one shared fp16 (S, Z) per group, write them at token offset n_quant[b], then
 * move buffer tokens [n_tokens, n_buf[b]) to the front of the buffer.
 *   n_tokens: multiple of group, <= every n_buf[b]; n_quant[b] + n_tokens <= q_cap.
 * The host arrays are not modified: afterwards the caller adds n_tokens to n_quant[b] and
 * subtracts it from n_buf[b].
 */
int qs_quantize_flush(const qs_cache *c, int32_t n_tokens, void *stream);

/*
 * QUANTIZE at prefill (Algorithm 1, prefill stage, where the two planes are first built): quantize
 * n_tokens tokens of caller-provided fp16 K / V, device [B][Hkv][src_stride_tokens][128], into the
 * planes at token offset n_quant[b].  n_tokens is a multiple of group.  The buffer is not touched.
 */
int qs_quantize_prefill(const qs_cache *c, const void *k_src, const void *v_src,
                        int64_t src_stride_tokens, int32_t n_tokens, void *stream);

/*
 * Append new tokens to the full-precision buffer (Appendix A: C_K = concat(C_K, c_k), likewise C_V;
 * Section 4.3.2: tokens generated during decoding go, in full precision, to the second half of the buffer):
 *   k_new, v_new : device fp16 [B][n_new][n_kv_heads][128]  (token-major, as a projection produces them)
 * are written to buffer rows [n_buf[b], n_buf[b] + n_new) of every sequence.  n_buf[b] + n_new must not
 * exceed buf_cap.  The host lengths are not modified (the caller adds n_new).  Rejecting drafted tokens
 * (Algorithm 1 REJECTCACHE) needs no call at all: the caller lowers n_buf[b].
 */
int qs_append(const qs_cache *c, const void *k_new, const void *v_new, int32_t n_new, void *stream);

/*
 * DRAFT attention (Algorithm 1; Section 4.2: the draft pass loads the upper 4-bit plane only):
 *   q   : device fp16 [B][1][n_q_heads][128]
 *   out : device fp16 [B][1][n_q_heads][128]
 * The query of sequence b attends the decoded upper plane of tokens [0, n_quant[b]) and buffer
 * tokens [0, n_buf[b]) (its own K/V must already be the last buffer token; Appendix A).
 * out = softmax(sm_scale * q K^T) V, sm_scale > 0 and finite (QS_ERR_RANGE otherwise).
 * Numerical domain (both attention calls): any finite fp16 q, K and V.  The 2e-3 accuracy of the outputs does
 * not depend on their magnitudes: a row's queries, the key scales of a group and the value scales met so far are
 * each brought into a fixed range by a power of two before they enter the matrix cores as fp16 numbers.
 * lse (device float [B][1][n_q_heads], natural log of the
 * softmax normaliser) is written if not NULL.
 */
int qs_attn_draft(const qs_cache *c, const void *q, void *out, float sm_scale,
                  void *workspace, size_t workspace_bytes, float *lse, void *stream);

/*
 * TARGET / verify attention (Algorithm 1; Section 4.2: the target pass loads both 4-bit planes and
 * combines them into the INT8 code):
 *   q   : device fp16 [B][nq][n_q_heads][128], 1 <= nq <= QS_MAX_NQ (nq = gamma + 1)
 *   out : device fp16 [B][nq][n_q_heads][128]
 * The nq tokens' K/V must already be the LAST nq buffer tokens.  Query i (0-based) attends all
 * quantized tokens (decoded from 16 C_U + C_L) and buffer tokens [0, n_buf[b] - nq + i].
 */
int qs_attn_verify(const qs_cache *c, const void *q, int32_t nq, void *out, float sm_scale,
                   void *workspace, size_t workspace_bytes, float *lse, void *stream);

/*
 * The two attention calls above for callers that can neither allocate device memory nor be handed a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * verify == 0: exactly qs_attn_draft (nq must be 1); verify == 1: exactly qs_attn_verify.  The split-K
 * partials go to an array of QS_STATIC_WS_BYTES that is part of the library's code object; every GPU the
 * library runs on holds its own copy from the first call on it until the process ends.  The call
 * allocates nothing and frees nothing.  Its first call on a device looks the array's address up
 * (hipGetSymbolAddress) and should therefore happen outside a stream capture.
 *   - QS_ERR_WORKSPACE if qs_workspace_bytes(c, nq) exceeds QS_STATIC_WS_BYTES (nothing is enqueued).
 *   - Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (two
 *     streams, two threads) race on it and corrupt each other's results; calls on one stream are ordered.
 *   - Nothing in the array has to start at zero: each call writes every partial before it reads it.
 */
int qs_attn_static(const qs_cache *c, const void *q, int32_t nq, int32_t verify, void *out,
                   float sm_scale, float *lse, void *stream);

/*
 * Inspection helper: expand the packed planes and metadata of tokens [0, n_tokens) of one unit
 * into plain arrays (device pointers, any may be NULL to skip):
 *   k_u, v_u : uint8 [n_tokens][128]      C_U       k_l, v_l : int8 [n_tokens][128]  C_L
 *   k_s, k_z : fp16  [n_tokens/G][D]      per-(group, channel) S, Z in channel order
 *   v_s, v_z : fp16  [n_tokens][D/G]      per-(token, value group) S, Z in token order
 * n_tokens is a multiple of group.
 */
int qs_export_codes(const qs_cache *c, int32_t b, int32_t kv_head, int32_t n_tokens,
                    void *k_u, void *k_l, void *k_s, void *k_z,
                    void *v_u, void *v_l, void *v_s, void *v_z, void *stream);

/*
 * ---- The draft model's linear layers: 4-bit weights (abstract; Section 4, first paragraph) ----
 * The draft model shares the target's architecture with its weights in INT4.  The paper names no quantizer for
 * them; this library applies the one of Section 4.2 (upper plane only): asymmetric round-to-nearest codes
 * C in [0, 15], w_hat = C S + Z, one fp16 pair (S, Z) per output row and QS_W4_GROUP consecutive input channels
 * (the group size of Section 5.1), Z = min, S = (max - min) / 15, S = 1 where that is zero, code decisions
 * in binary32 as for the cache.
 *
 * A layer y = x W^T with W [n_out][n_in]: n_out a multiple of 16, n_in a multiple of QS_W4_GROUP and at most 32768.
 * packed (device, caller-owned, qs_w4_bytes() bytes, 16-byte aligned; qs_w4_quantize is its only writer) holds the
 * weights in blocks of 16 output rows x 128 input channels, block (T, g) = tile T of rows, group g of channels,
 * numbered b = T*(n_in/128) + g, in two regions:
 *   codes, from byte 0, 1024 bytes per block at 1024*b: one 32-bit word per lane of a 64-lane wave
 *                 (lane = 16*a + r, a < 4, r < 16) and matrix-core step s < 4, at (lane*4 + s)*4: row 16*T + r,
 *                 input channels 128*g + 32*s + 8*a + i (i < 8), channel i in nibble (i&1)*4 + (i>>1)
 *   scales and zeros, from byte 1024*(n_out/16)*(n_in/128), 64 bytes per block at 64*b: for a < 4, at 16*a,
 *                 S of rows 16*T + 4*a .. + 3 (four fp16), then their Z (four fp16)
 * Error behaviour as above: negative code, nothing enqueued.  QS_ERR_SHAPE for sizes that are not multiples
 * as stated or m outside 1..QS_W4_MAX_ROWS, QS_ERR_NULL / QS_ERR_ALIGN for pointers.
 */
#define QS_W4_GROUP 128
#define QS_W4_MAX_ROWS 16
typedef struct {
  int32_t n_out, n_in;
  void *packed;
} qs_w4;

/* Bytes of `packed` for a layer of this size; 0 if the size is not supported. */
size_t qs_w4_bytes(int32_t n_out, int32_t n_in);

/* Quantizes w (device fp16 [n_out][n_in], row-major) into l->packed. */
int qs_w4_quantize(const qs_w4 *l, const void *w, void *stream);

/*
 * y[i][n] = sum_k x[i][k] w_hat[n][k] for i < m:  x device fp16 [m][n_in], y device fp16 [m][n_out],
 * 1 <= m <= QS_W4_MAX_ROWS (the draft's decode step is m = 1 per sequence).  Products of codes and inputs
 * are exact, sums are binary32, y is rounded to fp16 once.  Deterministic: a row's sum is formed in a fixed order.
 */
int qs_w4_linear(const qs_w4 *l, const void *x, int32_t m, void *y, void *stream);

/*
 * Inspection helper: codes uint8 [n_out][n_in], scale and zero fp16 [n_out][n_in/128] (device pointers, any
 * may be NULL to skip).
 */
int qs_w4_export(const qs_w4 *l, void *codes, void *scale, void *zero, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QUANTSPEC_H_ */
