/*
 * swiftkv.h - C ABI of libswiftkv: the SwiftKV prefill forward pass for a
 * Llama-style grouped-query decoder on one AMD MI355X (gfx950).
 *
 * Method (SwiftKV paper): prompt tokens run decoder layers 1..l in full
 * (Sec. 3.1); the residual stream after layer l then feeds the K/V projections
 * of every later layer j > l (Sec. 3.2, Eq. 2: KV_j = W_KV^j x_{l+1}), with
 * AcrossKV letting the first layer of each group of g consecutive later layers
 * compute the K/V the whole group shares (Sec. 3.3).  Only the last new token of
 * each sequence (and decode tokens) continues through layers l+1..L to give
 * logits (footnote of Sec. 3.2; forward-pass order of Sec. 3.5).  The KV cache
 * is paged (Sec. 3.5 names PagedAttention) and may be stored as FP8 e4m3
 * (Appendix B.1 combines SwiftKV with FP8 KV quantisation).
 *
 * Conventions for every call
 *  - "dev" pointers are device (HBM) pointers owned by the caller; "host"
 *    pointers are ordinary host memory read before the call returns.
 *  - The library allocates no device memory, ever: weights, cache, block
 *    tables, logits, the workspace of a call and the buffer that holds the
 *    re-arranged weight copies (pack_buf of swiftkv_create) are the caller's
 *    (one static device array: see swiftkv_op_gemm_rows_static).
 *    A context owns host memory only (tables, a small pinned staging ring for
 *    the per-call plan, HIP events).
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and the call returns without waiting for it, unless its
 *    comment says that it synchronises.
 *  - Return value: SWIFTKV_OK (0) or a negative error; swiftkv_last_error()
 *    then gives a thread-local message.  Outputs are unspecified after an error.
 *  - A context is not thread-safe: one call at a time per context.
 *  - All matrices are bf16, row-major [out_features, in_features].
 */
#ifndef SWIFTKV_H
#define SWIFTKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SWIFTKV_OK = 0,
  SWIFTKV_EINVAL = -1, /* bad shape / argument                                */
  SWIFTKV_ENOSPC = -2, /* workspace, pack buffer or block table too small     */
  SWIFTKV_EHIP = -3,   /* HIP runtime failure (message carries the HIP error) */
  SWIFTKV_EDATA = -4   /* device-side input check failed (token id or block id out of range) */
};

enum { SWIFTKV_KV_BF16 = 0, SWIFTKV_KV_FP8_E4M3 = 1 };
enum { SWIFTKV_SCALE_COMPUTE_ABSMAX = 0, SWIFTKV_SCALE_USE_GIVEN = 1, SWIFTKV_SCALE_PER_TOKEN = 2 };

#define SWIFTKV_BLOCK_SIZE 16 /* tokens per paged KV block (fixed) */

/* Decoder shape (Sec. 3.1: grouped-query attention, d_g | d_k).  Constraints
 * checked by swiftkv_create: head_dim is 64 or 128; n_q_heads / n_kv_heads is 1,
 * 2, 4 or 8; n_q_heads*head_dim and n_kv_heads*head_dim are multiples of 128;
 * hidden, ffn and vocab are multiples of 16. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rope_theta; /* RoPE base; rotate-half pairing (i, i + head_dim/2), no frequency rescaling */
  float rms_eps;
} swiftkv_model_cfg;

/* Model weights (Sec. 3.1: W_Q, W_K, W_V; plus the rest of a Llama layer).
 * Per-layer members are HOST arrays of n_layers dev pointers.  wk/wv of a later
 * layer that is not the first of its AcrossKV group are never read and may be
 * NULL (the paper discards them after distillation, Sec. 3.4).  The weights are
 * read by every call and never modified; they must outlive the context. */
typedef struct {
  const void *embed;          /* dev [vocab, hidden]                      */
  const void *const *norm1;   /* dev [hidden]   input RMSNorm gain        */
  const void *const *wq;      /* dev [n_q_heads*head_dim, hidden]         */
  const void *const *wk;      /* dev [n_kv_heads*head_dim, hidden]        */
  const void *const *wv;      /* dev [n_kv_heads*head_dim, hidden]        */
  const void *const *wo;      /* dev [hidden, n_q_heads*head_dim]         */
  const void *const *norm2;   /* dev [hidden]   post-attention RMSNorm    */
  const void *const *wgate;   /* dev [ffn, hidden]                        */
  const void *const *wup;     /* dev [ffn, hidden]                        */
  const void *const *wdown;   /* dev [hidden, ffn]                        */
  const void *final_norm;     /* dev [hidden]                             */
  const void *lm_head;        /* dev [vocab, hidden] (not tied to embed)  */
} swiftkv_weights;

/* Paged KV cache (Sec. 3.5; one cache layer per AcrossKV group, Sec. 3.3).
 * Element (cache layer c, kv in {0=K,1=V}, block, offset, head, dim) lives at
 *   ((((c*2 + kv)*n_blocks + block)*16 + offset)*n_kv_heads + head)*head_dim + dim.
 * Model layer j (1-based) uses cache layer j-1 for j <= l and
 * l + (j-l-1)/g for j > l, so n_cache_layers = l + (L-l)/g.  K is stored after
 * RoPE.  FP8 mode (Appendix B.1) stores OCP e4m3fn codes; value = code *
 * scales[c][kv][head], or, with per-token scales (the granularity Appendix B.1
 * uses), code * scales[c][kv][slot] with slot = block*16 + offset of the token. */
typedef struct {
  void *data;                  /* dev, bf16 (2 B) or e4m3 (1 B) elements, layout above     */
  float *scales;               /* dev fp32, FP8 only: [n_cache_layers][2][n_kv_heads], or
                                  [n_cache_layers][2][n_blocks*16] with PER_TOKEN          */
  const int32_t *block_tables; /* dev [n_seqs][max_blocks_per_seq] physical block ids      */
  const int32_t *context_lens; /* host [n_seqs] tokens of each sequence already cached     */
  int32_t n_cache_layers, n_blocks, block_size /* must be 16 */, max_blocks_per_seq;
  int32_t dtype;               /* SWIFTKV_KV_BF16 | SWIFTKV_KV_FP8_E4M3                     */
  int32_t scale_mode;          /* FP8: COMPUTE_ABSMAX writes scales = absmax/448 over the
                                  tokens this call stores (only when no sequence of the call
                                  has cached context: older codes would be read under the
                                  new scale); USE_GIVEN reads the caller's scales;
                                  PER_TOKEN writes, for every token this call stores, its own
                                  K and V scale (absmax over all KV heads / 448) and reads
                                  cached tokens with theirs                                */
} swiftkv_kv_cache;

typedef struct swiftkv_ctx swiftkv_ctx;

/* Size in bytes of the buffer swiftkv_create needs for its re-arranged weight
 * copies (no passage of the paper: an implementation detail of this library).
 * swiftkv_pack_bytes_min covers the weight-row tables and the operand of the
 * single fused K/V projection of Eq. 2 (the group leaders' [W_K;W_V], each with
 * its layer's input-norm gain folded in: (L-l)/g * 2*n_kv_heads*head_dim * hidden
 * bf16 elements).  swiftkv_pack_bytes adds, when hidden, n_q_heads*head_dim and
 * ffn are multiples of 256, copies of [W_Q;W_K;W_V], W_O, [W_gate;W_up] and
 * W_down of layers 1..l and of the fused operand in the register-fragment order
 * of the matrix instructions (about l * (2*hidden*q_dim + 2*hidden*kv_dim +
 * 3*hidden*ffn) bf16 elements: 7.3 GB for the 8B shape at l = 16, 70 GB for the
 * 70B shape at l = 40), which lets the large GEMMs load weights without
 * passing them through LDS (10-18 % faster); for other shapes both sizes are
 * equal.  Both return 0 for an invalid (cfg, l, g). */
size_t swiftkv_pack_bytes(const swiftkv_model_cfg *cfg, int32_t l, int32_t acrosskv_group);
size_t swiftkv_pack_bytes_min(const swiftkv_model_cfg *cfg, int32_t l, int32_t acrosskv_group);

/* Bind a model, the SwiftKV split l (1 <= l <= n_layers: number of layers the
 * prompt runs in full, Sec. 3.2) and the AcrossKV group size g >= 1 with
 * (n_layers - l) % g == 0 (Sec. 3.3; 1 = off).  pack_buf (dev, 256-byte aligned,
 * pack_bytes long, caller-owned, must outlive the context) receives the weight
 * copies described above: with pack_bytes >= swiftkv_pack_bytes() all of them,
 * with swiftkv_pack_bytes_min() <= pack_bytes < swiftkv_pack_bytes() only the
 * minimum (the large GEMMs then stage both operands through LDS), with less
 * the call fails with SWIFTKV_ENOSPC.  The packing kernels run on `stream`;
 * the call synchronises that stream before it returns.  Allocates no device
 * memory. */
int swiftkv_create(swiftkv_ctx **out, const swiftkv_model_cfg *cfg, const swiftkv_weights *w,
                   int32_t l, int32_t acrosskv_group, void *pack_buf, size_t pack_bytes, void *stream);
/* Releases the context's host memory and events (no passage).  The caller's
 * buffers are untouched; pending work of earlier calls must have finished. */
void swiftkv_destroy(swiftkv_ctx *ctx);

/* Bytes of dev workspace swiftkv_prefill needs for up to max_tokens new tokens
 * in up to max_seqs sequences with the given cache dtype, when no sequence
 * brings more than one new token on top of a cached context (no passage: the
 * activations of Sec. 3.1's layers plus the kernels' scratch live here). */
size_t swiftkv_workspace_bytes(const swiftkv_ctx *ctx, int64_t max_tokens, int32_t max_seqs,
                               int32_t kv_dtype);
/* The same when prompts may continue over a cached prefix (Sec. 3.1: prefill
 * in chunks): max_prefix_tokens bounds the sum of context_lens over the
 * sequences that bring more than one new token.  The extra space holds the
 * K rows and V^T columns of positions 0 .. context+new-1 of those sequences,
 * copied out of the paged cache once per layer for the attention kernel. */
size_t swiftkv_workspace_bytes_prefix(const swiftkv_ctx *ctx, int64_t max_tokens, int32_t max_seqs,
                                      int32_t kv_dtype, int64_t max_prefix_tokens);

/* SwiftKV prefill of a packed batch (Sec. 3.2 Eq. 2, Sec. 3.3, Sec. 3.5).
 *  token_ids  dev  int32 [T]  new tokens, sequence after sequence, T = sum(seq_lens)
 *  seq_lens   host int32 [n_seqs] new tokens per sequence (>= 1)
 *  kv         cache descriptor; kv->context_lens[b] cached tokens precede the new ones.
 *             context 0 with any number of new tokens = prompt prefill; context > 0
 *             with exactly one new token = decode token; context > 0 with more new
 *             tokens = the next chunk of a prompt whose earlier chunks are cached
 *             (new token i sits at position context + i and attends to the cached
 *             positions and to the new tokens up to itself; size the workspace with
 *             swiftkv_workspace_bytes_prefix, else SWIFTKV_ENOSPC).  An FP8 cache
 *             with SWIFTKV_SCALE_COMPUTE_ABSMAX and any context > 0 is rejected
 *             (SWIFTKV_EINVAL): use USE_GIVEN or PER_TOKEN there.
 *  logits_out dev fp32 [n_seqs, vocab]: logits of the last new token of each sequence.
 *  workspace  dev, 256-byte aligned; one call at a time per workspace.
 * Writes K/V of all T new tokens into every cache layer (layers <= l from their
 * own layer input, later cache layers from the layer-l output), then runs the
 * last token of each sequence through layers l+1..L.  Returns as soon as the
 * work is enqueued: the host arrays are consumed before the return, the plan
 * words travel through the context's pinned staging ring.  Token ids and block
 * ids outside their range are clamped on the device and flagged; the flag is
 * reported by swiftkv_export_plan, not by this call. */
int swiftkv_prefill(swiftkv_ctx *ctx, const int32_t *token_ids, const int32_t *seq_lens,
                    int32_t n_seqs, const swiftkv_kv_cache *kv, float *logits_out,
                    void *workspace, size_t workspace_bytes, void *stream);

/* The signature step alone (Eq. 2 + AcrossKV): from a given layer-l output
 * hidden_l (dev bf16 [T, hidden]) compute RMSNorm_j, the fused K/V projection of
 * all group leaders, RoPE on K and the paged scatter into cache layers l..  */
int swiftkv_kv_from_hidden(swiftkv_ctx *ctx, const void *hidden_l, const int32_t *seq_lens,
                           int32_t n_seqs, const swiftkv_kv_cache *kv, void *workspace,
                           size_t workspace_bytes, void *stream);

/* Simple early exit of the continuing tokens (Appendix B.4).  gain (dev bf16
 * [hidden]) and head (dev bf16 [vocab, hidden]) describe an extra language-model
 * head that reads the layer-l output of each sequence's last new token:
 * logits_ee = head * RMSNorm(h_l; gain).  After this call swiftkv_prefill
 * returns logits_ee for the sequences whose largest softmax probability
 * exceeds `threshold` (the paper uses 0.95) and the ordinary logits for the
 * others; the K/V cache is the same either way.  Both NULL switches it off.
 * The remaining layers still run for every row (they stream each weight once
 * whatever the number of rows, so dropping single rows saves nothing; a serving
 * loop that wants to skip them when every row exits has to look at the flags).
 * The pointers are kept, not copied.  Workspace sizes depend on this setting:
 * call swiftkv_workspace_bytes afterwards. */
int swiftkv_set_early_exit(swiftkv_ctx *ctx, const void *gain, const void *head, float threshold);
/* Exit flags (Appendix B.4) of the most recent swiftkv_prefill that used
 * `workspace`: dev int32 [n_seqs], 1 = the row's logits are the extra head's
 * (all 0 when off). */
int swiftkv_export_exit_flags(swiftkv_ctx *ctx, const void *workspace, int32_t *flags_out, void *stream);

/* Copy out the integer plan of the most recent swiftkv_prefill /
 * swiftkv_kv_from_hidden that used `workspace` (all dev outputs, any may be NULL):
 * slot_mapping int64 [T] (= block_table[b][p/16]*16 + p%16, the paged-cache
 * addressing Sec. 3.5 relies on), positions int32 [T], cu_seqlens int32
 * [n_seqs+1], last_rows int32 [n_seqs].  Synchronises the stream and returns
 * SWIFTKV_EDATA if the device-side input checks of that call failed. */
int swiftkv_export_plan(swiftkv_ctx *ctx, const void *workspace, int64_t *slot_mapping,
                        int32_t *positions, int32_t *cu_seqlens, int32_t *last_rows, void *stream);

/* Copy out the layer-l output x_{l+1} of Eq. 2 (rounded to bf16, dev [T, hidden])
 * left in `workspace` by the most recent swiftkv_prefill. */
int swiftkv_export_hidden(swiftkv_ctx *ctx, const void *workspace, void *hidden_out, void *stream);

/* ---- single operations, exposed for kernel-level checks and timing --------
 * (no passages: building blocks of the steps above) */

/* C[M,N] = A[M,K] * W[N,K]^T, bf16 inputs, fp32 accumulation.  out_f32 != 0
 * stores fp32, else bf16.  variant: 0 = pick by shape, 1 = 256x256 tile with
 * register-staged loads, 2 = 128x128 tile, 3 = weight-streaming kernel for
 * M <= 80 rows without a K split, 14 / 15 = the five-stage direct-to-LDS loop
 * with 4 / 8 waves (what 0 picks for M >= 1024, K % 64 == 0).  All dev. */
int swiftkv_op_gemm(const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K,
                    int32_t out_f32, int32_t variant, void *stream);
/* The same product (bf16 out) through the loop that takes the weights in matrix-
 * instruction fragment order straight into registers: W is first re-arranged
 * into w_packed (dev, N*K bf16 elements, caller-owned scratch), as swiftkv_create
 * does once per model.  Needs M >= 1024 and N, K multiples of 256. */
int swiftkv_op_gemm_packed(const void *A, const void *W, void *w_packed, void *C, int32_t M,
                           int32_t N, int32_t K, void *stream);
/* The weight-streaming kernels (M <= 80 rows: decode steps, the last-token tail)
 * with K split over up to 16 workgroups (slices of K whose activation rows a
 * workgroup keeps in LDS, or splits that keep all compute units streaming when
 * there are few column tiles); the splits' fp32 partial sums go through
 * `workspace` (dev, swiftkv_op_gemm_rows_workspace(M, N) bytes) and are added in
 * a fixed order. */
int swiftkv_op_gemm_rows(const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K,
                         int32_t out_f32, void *workspace, size_t workspace_bytes, void *stream);
size_t swiftkv_op_gemm_rows_workspace(int32_t M, int32_t N);
/* swiftkv_op_gemm_rows for callers that cannot allocate device memory or pass a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the K-split partial sums live in a static device array of
 * the library, 16 x 80 x 4096 fp32 = 21 MB per GPU, held until the process
 * ends.  Same kernels, same split, same summation order: results are bit-identical
 * to swiftkv_op_gemm_rows.  M <= 80 and N <= 4096, else SWIFTKV_EINVAL.  Calls no
 * allocating routine.  All calls on one GPU share the array (nothing in it has
 * to start at zero: a call writes every partial sum before it reads it), so
 * calls that overlap on one GPU -- different streams, different threads --
 * race; issue them on one stream or order them with events. */
int swiftkv_op_gemm_rows_static(const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K,
                                int32_t out_f32, void *stream);

/* Measurement aid: the rate (TFLOP/s, host double) at which the chip executes
 * nothing but v_mfma_f32_32x32x16_bf16 on the caller's data -- `operands` is
 * dev bf16, at least 16384 elements, e.g. values distributed like the model's
 * activations and weights -- with one 4-wave workgroup per CU, `iters` x 16
 * instructions per wave.  The chip is power-limited, so this rate depends on the
 * operand bits and is well below the data-sheet peak on random data.  `sink` is
 * dev scratch of at least 1 MB.  Synchronises the stream. */
int swiftkv_op_mfma_rate(const void *operands, int32_t iters, void *sink, size_t sink_bytes,
                         double *tflops_out, void *stream);

/* Causal grouped-query attention over packed fresh sequences (Sec. 3.1):
 * q dev bf16 [T, Hq*hd], k, v dev bf16 [T, Hkv*hd] (already rotated), out dev
 * bf16 [T, Hq*hd]; seq_lens host.  workspace as from
 * swiftkv_op_attention_workspace.  Synchronises the stream (its tables are
 * staged from pageable host memory). */
int swiftkv_op_attention_prefill(const void *q, const void *k, const void *v, void *out,
                                 const int32_t *seq_lens, int32_t n_seqs, int32_t n_q_heads,
                                 int32_t n_kv_heads, int32_t head_dim, void *workspace,
                                 size_t workspace_bytes, void *stream);
size_t swiftkv_op_attention_workspace(int64_t n_tokens, int32_t n_seqs, int32_t n_kv_heads,
                                      int32_t head_dim);

/* Single-query attention over a paged cache (what decode tokens and the last-
 * token tail run, Sec. 3.1 decoding phase / Sec. 3.5): row r of q (dev bf16
 * [n_rows, Hq*hd], already rotated) attends to keys 0 .. n_keys[r]-1 (host
 * array) of block-table row r; out dev bf16 [n_rows, Hq*hd].  cache_k / cache_v
 * are the K and V planes of ONE cache layer ([n_blocks*16][Hkv][hd], bf16 or
 * e4m3 codes); scale_k / scale_v are that layer's [Hkv] scales, or
 * [n_blocks*16] with scale_mode SWIFTKV_SCALE_PER_TOKEN (FP8 only).  An e4m3
 * cache is read by the matrix unit as codes (FP8-input MFMA).  workspace as
 * from swiftkv_op_attention_decode_workspace.  Synchronises the stream. */
int swiftkv_op_attention_decode(const void *q, void *out, const int32_t *n_keys, int32_t n_rows,
                                int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                const void *cache_k, const void *cache_v, int32_t kv_dtype,
                                int32_t scale_mode, const float *scale_k, const float *scale_v,
                                const int32_t *block_tables, int32_t max_blocks_per_seq,
                                int32_t n_blocks, void *workspace, size_t workspace_bytes, void *stream);
size_t swiftkv_op_attention_decode_workspace(int32_t n_rows, int32_t n_q_heads, int32_t head_dim);

/* Saturating round-to-nearest-even fp32 -> OCP e4m3fn of x[i]/scale, dev arrays
 * (the quantiser of the FP8 cache, Appendix B.1). */
int swiftkv_op_fp8_quantize(const float *x, float scale, uint8_t *codes, int64_t n, void *stream);

/* Executed floating-point operations of one prefill call of this ctx (GEMM and
 * attention parts; the accounting of the paper's Table 1: 2 per multiply-add,
 * only the work SwiftKV leaves), for throughput figures.  Host outputs. */
int swiftkv_flops(const swiftkv_ctx *ctx, const int32_t *seq_lens, const int32_t *context_lens,
                  int32_t n_seqs, double *gemm_flops, double *attn_flops);

/* Per-kernel-class device time of all swiftkv_prefill calls on this ctx since
 * swiftkv_set_timing last selected classes (which also clears the totals):
 * HIP events are recorded on each call's stream around every launch of the
 * selected classes (no passage: a measurement aid).  class_mask: bit c selects
 * class c, 0 switches timing off, SWIFTKV_TIME_ALL selects every class; any
 * other bit is SWIFTKV_EINVAL.  An event pair costs a few microseconds on the
 * stream, so a call with every class selected runs about 1 ms longer (a
 * decode step has ~450 launches); select only the class in question when the
 * call's own duration matters.  Classes:
 * 0 = QKV GEMM, 1 = O GEMM, 2 = gate/up GEMM, 3 = down GEMM (layers 1..l),
 * 4 = fused KV GEMM (Eq. 2), 5 = prefill attention, 6 = plan / embedding /
 * single-query attention of decode rows / gather, 7 = last-token tail,
 * 8 = RMSNorm and 1/rms kernels, 9 = KV commit (paged scatter, FP8 quantise,
 * V transpose).  ms_out / launches_out are host arrays of
 * SWIFTKV_N_TIME_CLASSES.  Reading waits for the last recorded event. */
#define SWIFTKV_N_TIME_CLASSES 10
#define SWIFTKV_TIME_ALL ((1 << SWIFTKV_N_TIME_CLASSES) - 1)
int swiftkv_set_timing(swiftkv_ctx *ctx, int32_t class_mask);
int swiftkv_get_timing(swiftkv_ctx *ctx, double ms_out[SWIFTKV_N_TIME_CLASSES],
                       int32_t launches_out[SWIFTKV_N_TIME_CLASSES]);

/* Thread-local message of the last failed call; library version string. */
const char *swiftkv_last_error(void);
const char *swiftkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SWIFTKV_H */
