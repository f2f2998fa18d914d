// Shared device helpers and launch declarations for libswiftkv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned short bf16_t;  // raw bf16 storage
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#define SKV_BLOCK 16

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even fp32 -> bf16 (hardware v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ bf16_t f32_to_bf16(float x) {
  __bf16 b = (__bf16)x;
  return __builtin_bit_cast(bf16_t, b);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}
__device__ __forceinline__ float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// Saturating RNE fp32 -> OCP e4m3fn (1-4-3, bias 7, max 448, no inf).
__device__ __forceinline__ uint8_t f32_to_e4m3fn(float x) {
  uint32_t u = __float_as_uint(x);
  uint32_t sign = (u >> 24) & 0x80u;
  float a = fabsf(x);
  if (!(a < 448.0f)) return (uint8_t)(sign | 0x7E);  // saturate (also NaN -> max; inputs are finite)
  uint32_t code;
  if (a < 0.015625f) {  // below 2^-6: subnormal grid of 2^-9; exact RNE via float add trick
    float r = a * 512.0f;                 // exact scaling
    float q = rintf(r);                   // RNE to integer 0..8
    code = (uint32_t)q;                   // 8 == smallest normal (0x08)
  } else {
    uint32_t au = __float_as_uint(a);
    uint32_t lsb = (au >> 20) & 1u;
    au += 0x7FFFFu + lsb;                 // RNE to 3 mantissa bits
    uint32_t e = (au >> 23) - 120u;       // rebias 127 -> 7
    uint32_t m = (au >> 20) & 7u;
    code = (e << 3) | m;
    if (code > 0x7E) code = 0x7E;
  }
  return (uint8_t)(sign | code);
}
__device__ __forceinline__ float e4m3fn_to_f32(uint8_t c) {
  uint32_t s = ((uint32_t)c & 0x80u) << 24;
  uint32_t e = (c >> 3) & 0xF, m = c & 7;
  float v = (e == 0) ? (float)m * 0.001953125f : __uint_as_float(((e + 120u) << 23) | (m << 20));
  return __uint_as_float(__float_as_uint(v) | s);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ------------------------------------------------------------------ GEMM ----
enum GemmEpi {
  EPI_STORE_BF16 = 0,  // C bf16 [M, ldc]
  EPI_STORE_F32 = 1,   // C fp32 [M, ldc]
  EPI_RESID = 2,       // C fp32 [M, ldc] += acc  (in place on the residual stream, which is kept in fp32)
  EPI_SWIGLU = 3,      // virtual N = 2*ffn in 16-row gate/up interleave; C bf16 [M, ffn]
  EPI_QKV = 4,         // rstd row scale, RoPE on q/k columns, q/k/v to separate row-major buffers
  EPI_KV = 5           // rstd row scale, RoPE on K columns, paged scatter (bf16) or staging (+absmax)
};

struct GemmParams {
  // activations: A [M, K] bf16 row-major, leading dimension lda
  const bf16_t *A;
  int64_t lda;
  int32_t M, N, K;  // N = (virtual) output columns
  // weights: table of device pointers, one per block of 16 (virtual) output rows,
  // each pointing at 16 rows of K contiguous bf16 with row stride ldw.
  // With wtab == nullptr the rows are simply W + n * ldw.
  const bf16_t *const *wtab;
  const bf16_t *W;
  int64_t ldw;
  // the same weights in MFMA fragment order (see launch_pack_w), or null: [N/32][K/16][64 lanes][8] bf16
  const bf16_t *wpack;
  // epilogue
  void *C;
  int64_t ldc;
  const float *rstd;      // [M] row scale 1/rms (QKV / KV / SWIGLU), may be null
  const float2 *cos_sin;  // [M][hd/2] (QKV / KV)
  int32_t head_dim, q_dim, kv_dim;
  bf16_t *q_out, *k_out, *v_out;  // QKV: [M,q_dim], [M,kv_dim], [M,kv_dim]
  // KV scatter
  bf16_t *cache;               // base of the bf16 cache
  const int64_t *slots;        // [M]
  int64_t cache_layer_stride;  // elements between cache layers (2 * n_blocks*16 * kv_dim)
  int64_t cache_kv_stride;     // elements between the K and V planes of a layer
  int32_t first_cache_layer;   // KV: cache layer of projection 0
  bf16_t *stage;               // KV FP8 mode: staging [M, N] bf16 instead of the cache
  uint32_t *amax;              // FP8: [n_cache_layers][2][Hkv] absmax bit patterns (atomicMax), or null
  // RESID in the packed-weight loop, optional: besides C += acc, write the operand of the next
  // projection, hb[m][n] = bf16(C_new[m][n] * hb_gain[n]) (hb_gain null = 1), and the sums of squares of
  // C_new over each 64-column block, ssq[m][n / 64] (N / 64 per row), from which 1/rms follows
  bf16_t *hb;
  const bf16_t *hb_gain;
  float *ssq;
  int32_t raster_gm;           // m tiles per rasterisation group (0 = default)
};

// Matrix-instruction rate on given operand data, nothing else in the loop: `iters` x 16 independent
// v_mfma_f32_32x32x16_bf16 per wave, 4 waves per workgroup, one workgroup per CU.
int launch_mfma_rate(const bf16_t *operands, float *sink, int32_t n_workgroups, int32_t iters, hipStream_t st);
int launch_gemm(const GemmParams &p, int epi, int variant, hipStream_t st);
bool gemm_uses_packed_weights(const GemmParams &p);

// skinny (weight-streaming) GEMM for M <= 80 rows
struct SkinnyParams {
  const bf16_t *A;  // [M, K] bf16 (already normalised where needed)
  int32_t M, N, K;
  const bf16_t *W;   // [N, K]
  const bf16_t *W2;  // SWIGLU: up-projection [N, K]
  void *C;           // bf16 [M,N] (STORE_BF16, SWIGLU) or fp32 (STORE_F32; RESID adds in place)
  float *partial;    // scratch for K-split partial sums, or null (then K is never split)
  size_t partial_bytes;   // its size; a split whose partial sums would not fit is not taken
  const bf16_t *const *wtab;   // instead of W: device table of N/16 pointers, entry i = rows 16i .. 16i+15 (row stride K),
                               // e.g. [W_Q; W_K; W_V] of a layer as one matrix
  int32_t *n_splits_out;       // HOST, or null.  Given (STORE_F32 / RESID only), a launch that splits K leaves the sum to its
                               // consumer: it writes the number of splits here, the splits' sums stay in `partial` as
                               // [split][M][N] fp32 and C is untouched; 1 = nothing left to do (C is final)
};
constexpr int SKINNY_MAX_SPLIT = 16;
constexpr size_t SKINNY_PARTIAL_BYTES = (size_t)SKINNY_MAX_SPLIT * 80 * 8192 * 4;   // the driver's scratch: 16 splits x 80 rows x 8192 columns fp32 (42 MB)
int launch_skinny(const SkinnyParams &p, int epi, hipStream_t st);

// Few-row batches (decode steps): the Q, K, V projections come out of the weight-streaming kernel as
// fp32; this step rotates q and k (rotate-half, angles of the row's position), rounds to bf16 once and,
// for an FP8 cache with computed scales, collects the absmax of the stored K and V values per KV head.
struct QkvFinishParams {
  const float *q32, *k32, *v32;   // rows of q_dim / kv_dim / kv_dim columns, row stride ld32 elements (0: dense)
  int32_t ld32;
  int32_t n_splits;               // > 1: the inputs are that many partial sums, T * ld32 elements apart, to be added in order
  bf16_t *q, *k, *v;
  int32_t T, n_q_heads, n_kv_heads, head_dim;
  const float2 *cos_sin;          // [T][hd/2]
  uint32_t *amax;                 // [2][Hkv] float bits of this cache layer, or null
};
int launch_qkv_finish(const QkvFinishParams &p, hipStream_t st);

// Simple early exit of the continuing tokens: flags[b] = 1 when the largest softmax probability of row b
// of `early` (fp32 [B, V]) exceeds `threshold`; select copies the flagged rows of `early` over `logits`.
int launch_early_exit_flags(const float *early, int32_t B, int32_t V, float threshold, int32_t *flags, hipStream_t st);
int launch_early_exit_select(const float *early, const int32_t *flags, float *logits, int32_t B, int32_t V, hipStream_t st);

// ------------------------------------------------------------- attention ----
struct QBlock {  // one 128-row query block of a sequence
  int32_t row0;   // packed row of the block's first query
  int32_t q0;     // position of that query inside the sequence (cached context included)
  int32_t n;      // keys available: cached context + new tokens
  int32_t seq_row0;  // row of the sequence's position 0 in the K buffer
  int32_t vt_col0;   // column of the sequence's position 0 in the V^T buffer
  int32_t q_last_row;  // packed row of the sequence's last query (stands in for rows past the end)
  int32_t pad[2];
};
struct AttnPrefillParams {
  const bf16_t *q, *k;  // [T, q_dim], [T, kv_dim]
  const bf16_t *vt;     // [kv_dim, vt_ld]  V transposed, sequences at 64-aligned columns
  int64_t vt_ld;
  bf16_t *out;          // [T, q_dim]
  const QBlock *qblocks;
  int32_t n_qblocks, n_q_heads, n_kv_heads, head_dim;
  int32_t *sched;       // nine device words, zero at launch (the kernel leaves them zero): next item of 8 queues, workgroups done
};
int launch_attention_prefill(const AttnPrefillParams &p, hipStream_t st);

struct DecodeRow {  // one single-query attention problem
  int32_t q_row;    // row in q buffer
  int32_t out_row;  // row in out buffer
  int32_t seq;      // sequence (block-table row)
  int32_t n_keys;   // keys 0..n_keys-1 are visible
  int32_t cs_row;   // row of cos/sin table to rotate q with, or -1
  int32_t pad[3];
};
struct AttnDecodeParams {
  const bf16_t *q;  // [*, q_dim]
  bf16_t *out;      // [*, q_dim]
  const DecodeRow *rows;
  int32_t n_rows, n_q_heads, n_kv_heads, head_dim;
  const void *cache_k, *cache_v;  // this cache layer's K and V planes [n_blocks*16][Hkv][hd]
  int32_t fp8;                     // 0 = bf16, 1 = e4m3 with per-head scales, 2 = e4m3 with per-slot scales
  const float *scale_k, *scale_v;  // [Hkv] (fp8 = 1) or [n_blocks*16] (fp8 = 2)
  const int32_t *block_tables;
  int32_t max_blocks_per_seq, n_blocks;
  const float2 *cos_sin;  // [T][hd/2]
  float *partial;         // [n_rows][Hq][n_split][hd + 2]
  int32_t n_split;
};
int launch_attention_decode(const AttnDecodeParams &p, hipStream_t st);

// ----------------------------------------------------------- elementwise ----
struct PlanParams {
  int32_t T, B, head_dim, n_blocks, max_blocks_per_seq, vocab;
  float rope_theta;
  const int32_t *cu_seqlens;    // dev [B+1]
  const int32_t *context_lens;  // dev [B]
  const int32_t *block_tables;  // dev
  const int32_t *token_ids;     // dev [T] (may be null)
  int32_t *positions, *seq_of, *last_rows, *err_flag;
  int64_t *slots;
  float2 *cos_sin;
};
int launch_plan(const PlanParams &p, hipStream_t st);
// The residual stream h is fp32 [rows, d] everywhere.
int launch_embed(const int32_t *ids, const bf16_t *E, float *h, int32_t T, int32_t d, int32_t vocab, hipStream_t st);
// rstd[t] = rsqrt(mean(h[t,:]^2) + eps) of bf16 rows (a layer-l output handed in by the caller)
int launch_rstd(const bf16_t *h, float *rstd, int32_t T, int32_t d, float eps, hipStream_t st);
// the same from per-block sums of squares ssq[T][n_blocks] written by the RESID epilogue, added in block order
int launch_rstd_from_ssq(const float *ssq, int32_t n_blocks, float *rstd, int32_t T, int32_t d, float eps, hipStream_t st);
// RMSNorm of fp32 rows into a bf16 GEMM operand.  rstd_out == null: out = bf16(h * rstd * gain).  Otherwise
// the row factor is left to the consumer's epilogue: out = bf16(h * gain) and rstd_out[row] = rstd.
// gain == null stands for a gain of one.
// With n_splits > 1 the rows first take the K-split sums a weight-streaming GEMM left behind: h[row] +=
// partial[0][row] + partial[1][row] + ... (partial: [n_splits][rows][d] fp32), written back to h.
int launch_rmsnorm_rows(float *h, const bf16_t *gain, bf16_t *out, int32_t rows, int32_t d, float eps, float *rstd_out, hipStream_t st,
                        const float *partial = nullptr, int32_t n_splits = 1);
int launch_gather_rows(const float *h, const int32_t *rows, float *out, int32_t n_rows, int32_t d, hipStream_t st);
int launch_f32_to_bf16(const float *x, bf16_t *out, int64_t n, hipStream_t st);
int launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t st);
// out[((n/32) * (K/16) + k/16) * 512 + ((k%16)/8 * 32 + n%32) * 8 + k%8] = W row n (through the optional
// 16-row block pointer table), element k.  N % 32 == 0, K % 16 == 0.  rope_hd == 128 (N % 128 == 0) takes the
// 32-row blocks of every 128 rows in the order 0, 2, 1, 3 (rotary partners side by side in a 64-row wave tile).
int launch_pack_w(const bf16_t *const *wtab, const bf16_t *W, int64_t ldw, int32_t N, int32_t K, int32_t rope_hd, bf16_t *out, hipStream_t st);
int launch_fold_gain(const bf16_t *W, const bf16_t *gain, bf16_t *out, int64_t rows, int32_t K, hipStream_t st);

struct KVTile {  // 64 consecutive new tokens of one sequence
  int32_t row0;     // packed row of first token
  int32_t n_valid;  // tokens present (1..64)
  int32_t vt_col0;  // V^T column of first token (64-aligned), or -1 when no V^T is wanted
  int32_t pad;
};
struct CommitParams {
  const KVTile *tiles;
  int32_t n_tiles, n_kv_heads, head_dim;
  bf16_t *k_src, *v_src;  // row-major [T, ld_src] (+ column offset applied by caller); fp8 writes dequantised values back
  int64_t ld_src;
  void *cache_k, *cache_v;  // planes of the destination cache layer
  const int64_t *slots;
  int32_t fp8, compute_scale, writeback;
  int32_t per_token;     // fp8 with one scale per cache slot: scales is [2][n_slots], set beforehand by the token-scale kernel
  int64_t n_slots;
  const uint32_t *amax;  // [2][Hkv] absmax bits of this cache layer (fp8 compute mode)
  float *scales;         // [2][Hkv] of this cache layer (fp8), or [2][n_slots]
  bf16_t *vt;            // [kv_dim, vt_ld] or null
  int64_t vt_ld;
};
int launch_kv_commit(const CommitParams &p, hipStream_t st);

// FP8 cache with per-token scales (Appendix B.1): scale of a token = absmax of its K (V) row over all
// KV heads / 448, stored at the token's cache slot.
struct TokenScaleParams {
  const bf16_t *k_src, *v_src;   // row-major [T, ld_src]
  int64_t ld_src;
  int32_t T, kv_dim;
  const int64_t *slots;
  float *scales;                 // [2][n_slots] of this cache layer
  int64_t n_slots;
};
int launch_token_scales(const TokenScaleParams &p, hipStream_t st);

// Prompt chunks over a cached prefix: the prefill attention reads contiguous K rows and V^T columns,
// so positions 0 .. context+new-1 of such sequences are copied out of the paged cache first.
struct GatherTile {  // 64 consecutive positions of one sequence
  int32_t seq;       // block-table row
  int32_t pos0;      // first position
  int32_t n_valid;   // positions present (the rest of the V^T columns is zero filled)
  int32_t k_row0;    // destination row of pos0 in the K buffer
  int32_t vt_col0;   // destination column of pos0 in the V^T buffer (64-aligned)
  int32_t pad[3];
};
struct GatherParams {
  const GatherTile *tiles;
  int32_t n_tiles, n_kv_heads, head_dim;
  const void *cache_k, *cache_v;   // planes of the cache layer [n_blocks*16][Hkv][hd], bf16 or e4m3 codes
  int32_t fp8;                     // 0 = bf16, 1 = e4m3 with per-head scales, 2 = e4m3 with per-slot scales
  const float *scales;             // [2][Hkv] of this cache layer (fp8 = 1) or [2][n_blocks*16] (fp8 = 2)
  const int32_t *block_tables;
  int32_t max_blocks_per_seq, n_blocks;
  bf16_t *k_dst;                   // [rows, kv_dim]
  bf16_t *vt;                      // [kv_dim, vt_ld]
  int64_t vt_ld;
};
int launch_kv_gather(const GatherParams &p, hipStream_t st);
int launch_fp8_quantize(const float *x, float scale, uint8_t *codes, int64_t n, hipStream_t st);
int launch_decode_combine(const float *partial, bf16_t *out, const DecodeRow *rows, int32_t n_rows,
                          int32_t n_q_heads, int32_t head_dim, int32_t n_split, hipStream_t st);
