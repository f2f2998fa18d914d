// HBM-bound kernels of the SwiftKV prefill path: integer plan + RoPE table,
// embedding gather, row rstd, RMSNorm of a few rows, row gather, KV commit
// (paged scatter, FP8 quantise, V transpose), split-KV combine.
#include "common.h"

// ---------------------------------------------------------------- plan -----
// One thread per (new token, rotary pair): sequence by binary search in
// cu_seqlens, absolute position, paged slot = block_table[b][p/16]*16 + p%16
// (written by the token's first thread), and the RoPE angle table
// cos/sin(p * theta^(-2i/hd)) formed in double precision.
__global__ void plan_kernel(PlanParams p) {
  const int half = p.head_dim / 2;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid < p.B) p.last_rows[gid] = p.cu_seqlens[gid + 1] - 1;
  const int t = (int)(gid / half), i = (int)(gid % half);
  if (t >= p.T) return;
  int lo = 0, hi = p.B - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (p.cu_seqlens[mid] <= t) lo = mid; else hi = mid - 1;
  }
  const int b = lo;
  const int pos = p.context_lens[b] + (t - p.cu_seqlens[b]);
  if (i == 0) {
    int blk = p.block_tables[(int64_t)b * p.max_blocks_per_seq + pos / SKV_BLOCK];
    if (blk < 0 || blk >= p.n_blocks) {  // never let a bad table turn into a wild store
      atomicOr(p.err_flag, 1);
      blk = 0;
    }
    if (p.token_ids) {
      int id = p.token_ids[t];
      if (id < 0 || id >= p.vocab) atomicOr(p.err_flag, 2);
    }
    p.positions[t] = pos;
    p.seq_of[t] = b;
    p.slots[t] = (int64_t)blk * SKV_BLOCK + pos % SKV_BLOCK;
  }
  const double inv_freq = pow((double)p.rope_theta, -2.0 * (double)i / (double)p.head_dim);
  const double ang = (double)pos * inv_freq;
  p.cos_sin[(int64_t)t * half + i] = make_float2((float)cos(ang), (float)sin(ang));
}
int launch_plan(const PlanParams &p, hipStream_t st) {
  const int64_t n = std::max<int64_t>((int64_t)p.T * (p.head_dim / 2), p.B);
  hipLaunchKernelGGL(plan_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p);
  return 0;
}

// --------------------------------------------------------------- embed -----
// h[t, :] = E[id[t], :] widened to fp32 (the residual stream is kept in fp32).
__global__ void embed_kernel(const int32_t *ids, const uint4 *E, float4 *h, int T, int chunks, int vocab) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)T * chunks) return;
  int t = (int)(i / chunks), c = (int)(i % chunks);
  int id = ids[t];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  const uint4 u = E[(int64_t)id * chunks + c];
  h[2 * i] = make_float4(bf16lo(u.x), bf16hi(u.x), bf16lo(u.y), bf16hi(u.y));
  h[2 * i + 1] = make_float4(bf16lo(u.z), bf16hi(u.z), bf16lo(u.w), bf16hi(u.w));
}
int launch_embed(const int32_t *ids, const bf16_t *E, float *h, int32_t T, int32_t d, int32_t vocab, hipStream_t st) {
  int chunks = d / 8;
  int64_t n = (int64_t)T * chunks;
  hipLaunchKernelGGL(embed_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ids, (const uint4 *)E, (float4 *)h, T, chunks, vocab);
  return 0;
}

// ---------------------------------------------------------------- rstd -----
// rstd[t] = rsqrt(mean(h[t,:]^2) + eps); one wave per row.
__global__ void rstd_kernel(const uint4 *h, float *rstd, int T, int chunks, float eps, float inv_d) {
  int row = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  int lane = threadIdx.x & 63;
  if (row >= T) return;
  const uint4 *r = h + (int64_t)row * chunks;
  float s = 0.f;
  for (int c = lane; c < chunks; c += 64) {
    uint4 u = r[c];
    float a;
    a = bf16lo(u.x); s += a * a; a = bf16hi(u.x); s += a * a;
    a = bf16lo(u.y); s += a * a; a = bf16hi(u.y); s += a * a;
    a = bf16lo(u.z); s += a * a; a = bf16hi(u.z); s += a * a;
    a = bf16lo(u.w); s += a * a; a = bf16hi(u.w); s += a * a;
  }
  s = wave_sum(s);
  if (lane == 0) rstd[row] = rsqrtf(s * inv_d + eps);
}
int launch_rstd(const bf16_t *h, float *rstd, int32_t T, int32_t d, float eps, hipStream_t st) {
  hipLaunchKernelGGL(rstd_kernel, dim3((T + 3) / 4), dim3(256), 0, st, (const uint4 *)h, rstd, T, d / 8, eps, 1.0f / (float)d);
  return 0;
}

// 1/rms from the per-block sums of squares the residual epilogue of the packed-weight GEMM leaves:
// ssq[t][b], b < n_blocks (a multiple of 4), added in block order (fixed order: results do not change
// from run to run).  One thread per row; its loads are independent of each other.
__global__ void rstd_from_ssq_kernel(const float4 *ssq, int n_quads, float *rstd, int T, float eps, float inv_d) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float4 *r = ssq + (int64_t)t * n_quads;
  float s = 0.f;
  for (int q0 = 0; q0 < n_quads; q0 += 8) {
    float4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = q0 + i < n_quads ? r[q0 + i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 8; ++i) { s += v[i].x; s += v[i].y; s += v[i].z; s += v[i].w; }
  }
  rstd[t] = rsqrtf(s * inv_d + eps);
}
int launch_rstd_from_ssq(const float *ssq, int32_t n_blocks, float *rstd, int32_t T, int32_t d, float eps, hipStream_t st) {
  hipLaunchKernelGGL(rstd_from_ssq_kernel, dim3((T + 63) / 64), dim3(64), 0, st, (const float4 *)ssq, n_blocks / 4, rstd, T, eps, 1.0f / (float)d);
  return 0;
}

// ------------------------------------------------------- RMSNorm of rows ----
// fp32 rows -> bf16 GEMM operand; one wave per row.  With rstd_out the row factor is left to the
// consumer: out = bf16(h * gain), rstd_out[row] = 1/rms; else out = bf16(h * 1/rms * gain).
__device__ __forceinline__ uint2 norm4(const float4 u, const float rs, const bf16_t *gain, int c) {
  float g0 = 1.f, g1 = 1.f, g2 = 1.f, g3 = 1.f;
  if (gain) {
    const uint2 g = *(const uint2 *)(gain + 4 * c);
    g0 = bf16lo(g.x); g1 = bf16hi(g.x); g2 = bf16lo(g.y); g3 = bf16hi(g.y);
  }
  return make_uint2(pack_bf16x2(u.x * rs * g0, u.y * rs * g1), pack_bf16x2(u.z * rs * g2, u.w * rs * g3));
}
__global__ void rmsnorm_rows_kernel(const float4 *h, const bf16_t *gain, uint2 *out, int rows, int chunks, float eps, float inv_d, float *rstd_out) {
  int row = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float4 *r = h + (int64_t)row * chunks;
  float s = 0.f;
  for (int c = lane; c < chunks; c += 64) {
    const float4 u = r[c];
    s += u.x * u.x; s += u.y * u.y; s += u.z * u.z; s += u.w * u.w;
  }
  s = wave_sum(s);
  const float rs = rsqrtf(s * inv_d + eps);
  if (rstd_out && lane == 0) rstd_out[row] = rs;
  const float f = rstd_out ? 1.f : rs;
  for (int c = lane; c < chunks; c += 64) out[(int64_t)row * chunks + c] = norm4(r[c], f, gain, c);
}
// Single-pass variant: the row (d = 256 * CH elements) stays in registers between the reduction and the
// scaling; the gains are requested together with the row (asked for only after the reduction they were a
// second memory latency, which is most of the time of the few-row launches of decode steps and the tail).
template <int CH>
__global__ __launch_bounds__(256) void rmsnorm_rows_reg_kernel(const float4 *h, const bf16_t *gain, uint2 *out, int rows, float eps, float inv_d, float *rstd_out) {
  const int row = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float4 *r = h + (int64_t)row * (CH * 64);
  float4 u[CH];
  uint2 g[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) u[i] = r[i * 64 + lane];
#pragma unroll
  for (int i = 0; i < CH; ++i) g[i] = gain ? *(const uint2 *)(gain + 4 * (i * 64 + lane)) : make_uint2(0x3f803f80u, 0x3f803f80u);   // bf16 ones
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < CH; ++i) { s += u[i].x * u[i].x; s += u[i].y * u[i].y; s += u[i].z * u[i].z; s += u[i].w * u[i].w; }
  s = wave_sum(s);
  const float rs = rsqrtf(s * inv_d + eps);
  if (rstd_out && lane == 0) rstd_out[row] = rs;
  const float f = rstd_out ? 1.f : rs;
#pragma unroll
  for (int i = 0; i < CH; ++i)
    out[(int64_t)row * (CH * 64) + i * 64 + lane] =
        make_uint2(pack_bf16x2(u[i].x * f * bf16lo(g[i].x), u[i].y * f * bf16hi(g[i].x)), pack_bf16x2(u[i].z * f * bf16lo(g[i].y), u[i].w * f * bf16hi(g[i].y)));
}
// Few rows (decode steps, the tail): one workgroup of four waves per row, d = 1024 * CQ.  With n_splits > 1
// the row first takes the sums of the K splits a weight-streaming GEMM left in `partial` ([n_splits][rows][d]
// fp32): the splits are added in order, then to the row, which is written back.  The sum of squares is added
// over a lane's values in order, then over the wave, then over the four waves in order.
template <int CQ>
__global__ __launch_bounds__(256) void rmsnorm_row_wg_kernel(float4 *h, const bf16_t *gain, uint2 *out, int rows, float eps, float inv_d,
                                                             float *rstd_out, const float4 *partial, int n_splits) {
  __shared__ float red[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  float4 *r = h + (int64_t)row * (CQ * 256);
  float4 u[CQ];
  uint2 g[CQ];
#pragma unroll
  for (int i = 0; i < CQ; ++i) u[i] = r[i * 256 + tid];
#pragma unroll
  for (int i = 0; i < CQ; ++i) g[i] = gain ? *(const uint2 *)(gain + 4 * (i * 256 + tid)) : make_uint2(0x3f803f80u, 0x3f803f80u);
  if (n_splits > 1) {
    float4 sum[CQ];
#pragma unroll
    for (int i = 0; i < CQ; ++i) sum[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 *pr = partial + (int64_t)row * (CQ * 256) + tid;
    const int64_t step = (int64_t)rows * (CQ * 256);
    int ks = 0;
    for (; ks + 2 <= n_splits; ks += 2) {   // two splits' loads in flight, added in split order
      float4 v0[CQ], v1[CQ];
#pragma unroll
      for (int i = 0; i < CQ; ++i) { v0[i] = pr[ks * step + i * 256]; v1[i] = pr[(ks + 1) * step + i * 256]; }
#pragma unroll
      for (int i = 0; i < CQ; ++i) {
        sum[i].x += v0[i].x; sum[i].y += v0[i].y; sum[i].z += v0[i].z; sum[i].w += v0[i].w;
        sum[i].x += v1[i].x; sum[i].y += v1[i].y; sum[i].z += v1[i].z; sum[i].w += v1[i].w;
      }
    }
    if (ks < n_splits) {
#pragma unroll
      for (int i = 0; i < CQ; ++i) {
        const float4 v = pr[ks * step + i * 256];
        sum[i].x += v.x; sum[i].y += v.y; sum[i].z += v.z; sum[i].w += v.w;
      }
    }
#pragma unroll
    for (int i = 0; i < CQ; ++i) {
      u[i].x += sum[i].x; u[i].y += sum[i].y; u[i].z += sum[i].z; u[i].w += sum[i].w;
      r[i * 256 + tid] = u[i];
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < CQ; ++i) { s += u[i].x * u[i].x; s += u[i].y * u[i].y; s += u[i].z * u[i].z; s += u[i].w * u[i].w; }
  s = wave_sum(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  s = ((red[0] + red[1]) + red[2]) + red[3];
  const float rs = rsqrtf(s * inv_d + eps);
  if (rstd_out && tid == 0) rstd_out[row] = rs;
  const float f = rstd_out ? 1.f : rs;
#pragma unroll
  for (int i = 0; i < CQ; ++i)
    out[(int64_t)row * (CQ * 256) + i * 256 + tid] =
        make_uint2(pack_bf16x2(u[i].x * f * bf16lo(g[i].x), u[i].y * f * bf16hi(g[i].x)), pack_bf16x2(u[i].z * f * bf16lo(g[i].y), u[i].w * f * bf16hi(g[i].y)));
}
// the K-split sums of a weight-streaming GEMM added into fp32 rows (for row widths the kernel above does not cover)
__global__ void add_splits_kernel(float4 *h, const float4 *partial, int64_t n4, int n_splits) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int ks = 0; ks < n_splits; ++ks) {
    const float4 v = partial[(int64_t)ks * n4 + i];
    sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
  }
  float4 u = h[i];
  u.x += sum.x; u.y += sum.y; u.z += sum.z; u.w += sum.w;
  h[i] = u;
}
int launch_rmsnorm_rows(float *h, const bf16_t *gain, bf16_t *out, int32_t rows, int32_t d, float eps, float *rstd_out, hipStream_t st,
                        const float *partial, int32_t n_splits) {
  if (rows <= 0) return 0;
  const dim3 grid((rows + 3) / 4), block(256);
  const float inv_d = 1.0f / (float)d;
  if (rows <= 256 && d % 1024 == 0 && d / 1024 <= 8) {   // few rows: a workgroup per row, K splits added on the way
#define SKV_RMS_WG(CQ_)                                                                                            \
  case CQ_:                                                                                                        \
    hipLaunchKernelGGL(rmsnorm_row_wg_kernel<CQ_>, dim3(rows), block, 0, st, (float4 *)h, gain, (uint2 *)out, rows, eps, inv_d, rstd_out, \
                       (const float4 *)partial, n_splits);                                                        \
    return 0;
    switch (d / 1024) {
      SKV_RMS_WG(1) SKV_RMS_WG(2) SKV_RMS_WG(3) SKV_RMS_WG(4) SKV_RMS_WG(5) SKV_RMS_WG(6) SKV_RMS_WG(7) SKV_RMS_WG(8)
      default: break;
    }
#undef SKV_RMS_WG
  }
  if (n_splits > 1) {   // otherwise: the splits in a pass of their own
    const int64_t n4 = (int64_t)rows * d / 4;
    hipLaunchKernelGGL(add_splits_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, (float4 *)h, (const float4 *)partial, n4, n_splits);
  }
#define SKV_RMS_CASE(CH_)                                                                                          \
  case CH_:                                                                                                        \
    hipLaunchKernelGGL(rmsnorm_rows_reg_kernel<CH_>, grid, block, 0, st, (const float4 *)h, gain, (uint2 *)out, rows, eps, inv_d, rstd_out); \
    return 0;
  if (d % 256 == 0) {
    switch (d / 256) {
      SKV_RMS_CASE(1) SKV_RMS_CASE(2) SKV_RMS_CASE(4) SKV_RMS_CASE(8) SKV_RMS_CASE(16) SKV_RMS_CASE(20) SKV_RMS_CASE(24) SKV_RMS_CASE(32)
      default: break;
    }
  }
#undef SKV_RMS_CASE
  hipLaunchKernelGGL(rmsnorm_rows_kernel, grid, block, 0, st, (const float4 *)h, gain, (uint2 *)out, rows, d / 4, eps, inv_d, rstd_out);
  return 0;
}

// ------------------------------------------- fold a norm gain into weights ----
// out[n, k] = bf16(W[n, k] * gain[k]): RMSNorm_j(x) W^T = rstd(x) * (x (W diag(g_j))^T), so the
// per-layer gain can live in the weights and only the row scale rstd is left for the GEMM epilogue.
__global__ void fold_gain_kernel(const uint4 *W, const uint4 *gain, uint4 *out, int64_t n_chunks, int chunks_per_row) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_chunks) return;
  uint4 u = W[i], g = gain[i % chunks_per_row], o;
  o.x = pack_bf16x2(bf16lo(u.x) * bf16lo(g.x), bf16hi(u.x) * bf16hi(g.x));
  o.y = pack_bf16x2(bf16lo(u.y) * bf16lo(g.y), bf16hi(u.y) * bf16hi(g.y));
  o.z = pack_bf16x2(bf16lo(u.z) * bf16lo(g.z), bf16hi(u.z) * bf16hi(g.z));
  o.w = pack_bf16x2(bf16lo(u.w) * bf16lo(g.w), bf16hi(u.w) * bf16hi(g.w));
  out[i] = o;
}
int launch_fold_gain(const bf16_t *W, const bf16_t *gain, bf16_t *out, int64_t rows, int32_t K, hipStream_t st) {
  int64_t n = rows * (K / 8);
  hipLaunchKernelGGL(fold_gain_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const uint4 *)W, (const uint4 *)gain, (uint4 *)out, n, K / 8);
  return 0;
}

// -------------------------------------------------------------- gather -----
__global__ void gather_rows_kernel(const float4 *h, const int32_t *rows, float4 *out, int n_rows, int chunks) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)n_rows * chunks) return;
  int r = (int)(i / chunks), c = (int)(i % chunks);
  out[i] = h[(int64_t)rows[r] * chunks + c];
}
int launch_gather_rows(const float *h, const int32_t *rows, float *out, int32_t n_rows, int32_t d, hipStream_t st) {
  int chunks = d / 4;
  int64_t n = (int64_t)n_rows * chunks;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const float4 *)h, rows, (float4 *)out, n_rows, chunks);
  return 0;
}

__global__ void f32_to_bf16_kernel(const float4 *x, uint2 *out, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const float4 u = x[i];
  out[i] = make_uint2(pack_bf16x2(u.x, u.y), pack_bf16x2(u.z, u.w));
}
int launch_f32_to_bf16(const float *x, bf16_t *out, int64_t n, hipStream_t st) {   // n % 4 == 0
  if (n <= 0) return 0;
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st, (const float4 *)x, (uint2 *)out, n / 4);
  return 0;
}

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
// One 16-byte chunk per thread: chunk id = ((block * K/16 + k16) * 64 + lane), lane = g*32 + l32.
// rope_hd == 128: inside every group of 128 rows (one head) the 32-row blocks are taken in the order
// 0, 2, 1, 3, so that a 64-row wave tile holds a block of the first half of the head next to its
// rotary partner block of the second half.
__global__ void pack_w_kernel(const bf16_t *const *wtab, const bf16_t *W, int64_t ldw, int32_t N, int32_t K, int32_t rope_hd, uint4 *out) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n_chunks = (int64_t)N * K / 8;
  if (id >= n_chunks) return;
  const int lane = (int)(id & 63);
  const int64_t frag = id >> 6;
  const int k16 = (int)(frag % (K / 16));
  int block = (int)(frag / (K / 16));
  if (rope_hd == 128) {
    const int b = block & 3;
    block = (block & ~3) | (b == 1 ? 2 : b == 2 ? 1 : b);
  }
  const int n = block * 32 + (lane & 31), k = k16 * 16 + (lane >> 5) * 8;
  const bf16_t *row = wtab ? wtab[n >> 4] + (int64_t)(n & 15) * ldw : W + (int64_t)n * ldw;
  const uint4 u = *(const uint4 *)(row + k);
  out[id] = u;
}
int launch_pack_w(const bf16_t *const *wtab, const bf16_t *W, int64_t ldw, int32_t N, int32_t K, int32_t rope_hd, bf16_t *out, hipStream_t st) {
  const int64_t n_chunks = (int64_t)N * K / 8;
  if (n_chunks <= 0) return 0;
  hipLaunchKernelGGL(pack_w_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st, wtab, W, ldw, N, K, rope_hd, (uint4 *)out);
  return 0;
}
int launch_fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t st) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
  return 0;
}

// ----------------------------------------------------------- KV commit -----
// One workgroup per (64-token tile, KV head).  Reads the tile's K and V rows
// (row-major, already rotated), stores them at their paged slots as bf16 or as
// e4m3 codes of x/scale, optionally writes the dequantised values back (so that
// attention sees exactly what the cache holds) and writes V transposed
// ([dim][token], 64-aligned columns, zero padded) for the prefill attention.
template <int HD>
__global__ __launch_bounds__(256) void kv_commit_kernel(CommitParams p) {
  constexpr int CH = HD / 8;  // 16-byte chunks per row
  __shared__ bf16_t sv[64][HD + 8];
  const KVTile tile = p.tiles[blockIdx.x];
  const int head = blockIdx.y;
  const int tid = threadIdx.x;
  float sk = 1.f, svs = 1.f, isk = 1.f, isv = 1.f;
  if (p.fp8 && !p.per_token) {
    if (p.compute_scale) {
      sk = fmaxf(__uint_as_float(p.amax[head]), 1e-12f) / 448.0f;
      svs = fmaxf(__uint_as_float(p.amax[p.n_kv_heads + head]), 1e-12f) / 448.0f;
      if (blockIdx.x == 0 && tid == 0) {
        p.scales[head] = sk;
        p.scales[p.n_kv_heads + head] = svs;
      }
    } else {
      sk = p.scales[head];
      svs = p.scales[p.n_kv_heads + head];
    }
  }
  (void)isk; (void)isv;
  const int kv_dim = p.n_kv_heads * HD;
  // everything this thread reads is requested before its first store (loads and stores share one
  // counter: a load issued after a store would wait for that store to reach memory)
  constexpr int NI = 64 * CH / 256;
  uint4 kin[NI], vin[NI];
  int64_t slot_in[NI];
  float sk_in[NI], sv_in[NI];
#pragma unroll
  for (int ii = 0; ii < NI; ++ii) {
    const int i = tid + ii * 256, r = i / CH, c = i % CH;
    kin[ii] = make_uint4(0, 0, 0, 0); vin[ii] = make_uint4(0, 0, 0, 0);
    slot_in[ii] = 0; sk_in[ii] = sk; sv_in[ii] = svs;
    if (r < tile.n_valid) {
      const int64_t row = tile.row0 + r;
      kin[ii] = *(const uint4 *)(p.k_src + row * p.ld_src + head * HD + c * 8);
      vin[ii] = *(const uint4 *)(p.v_src + row * p.ld_src + head * HD + c * 8);
      if (p.cache_k) slot_in[ii] = p.slots[row];
      if (p.per_token) { sk_in[ii] = p.scales[p.slots[row]]; sv_in[ii] = p.scales[p.n_slots + p.slots[row]]; }
    }
  }
#pragma unroll
  for (int ii = 0; ii < NI; ++ii) {
    const int i = tid + ii * 256;
    int r = i / CH, c = i % CH;
    uint4 kq = kin[ii], vq = vin[ii];
    if (r < tile.n_valid) {
      int64_t row = tile.row0 + r;
      bf16_t *kp = p.k_src + row * p.ld_src + head * HD + c * 8;
      bf16_t *vp = p.v_src + row * p.ld_src + head * HD + c * 8;
      int64_t dst = (slot_in[ii] * p.n_kv_heads + head) * HD + c * 8;
      sk = sk_in[ii]; svs = sv_in[ii];
      if (!p.cache_k) {
        // no cache wanted (stand-alone attention): only V^T is produced
      } else if (!p.fp8) {
        *(uint4 *)((bf16_t *)p.cache_k + dst) = kq;
        *(uint4 *)((bf16_t *)p.cache_v + dst) = vq;
      } else {
        uint32_t kw[4] = {kq.x, kq.y, kq.z, kq.w}, vw[4] = {vq.x, vq.y, vq.z, vq.w};
        uint32_t kc[2] = {0, 0}, vc[2] = {0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint8_t k0 = f32_to_e4m3fn(bf16lo(kw[e]) / sk), k1 = f32_to_e4m3fn(bf16hi(kw[e]) / sk);
          uint8_t v0 = f32_to_e4m3fn(bf16lo(vw[e]) / svs), v1 = f32_to_e4m3fn(bf16hi(vw[e]) / svs);
          kc[e / 2] |= ((uint32_t)k0 | ((uint32_t)k1 << 8)) << ((e & 1) * 16);
          vc[e / 2] |= ((uint32_t)v0 | ((uint32_t)v1 << 8)) << ((e & 1) * 16);
          kw[e] = pack_bf16x2(e4m3fn_to_f32(k0) * sk, e4m3fn_to_f32(k1) * sk);
          vw[e] = pack_bf16x2(e4m3fn_to_f32(v0) * svs, e4m3fn_to_f32(v1) * svs);
        }
        *(uint2 *)((uint8_t *)p.cache_k + dst) = make_uint2(kc[0], kc[1]);
        *(uint2 *)((uint8_t *)p.cache_v + dst) = make_uint2(vc[0], vc[1]);
        kq = make_uint4(kw[0], kw[1], kw[2], kw[3]);
        vq = make_uint4(vw[0], vw[1], vw[2], vw[3]);
        if (p.writeback) {
          *(uint4 *)kp = kq;
          *(uint4 *)vp = vq;
        }
      }
    }
    if (p.vt) {
      uint32_t w[4] = {vq.x, vq.y, vq.z, vq.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sv[r][c * 8 + 2 * e] = (bf16_t)(w[e] & 0xffff);
        sv[r][c * 8 + 2 * e + 1] = (bf16_t)(w[e] >> 16);
      }
    }
  }
  if (!p.vt || tile.vt_col0 < 0) return;
  __syncthreads();
  // V^T: thread writes 8 consecutive tokens of one dim (16 bytes)
  for (int i = tid; i < HD * 8; i += 256) {
    int d = i / 8, tc = i % 8;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (uint32_t)sv[tc * 8 + 2 * e][d] | ((uint32_t)sv[tc * 8 + 2 * e + 1][d] << 16);
    *(uint4 *)(p.vt + (int64_t)(head * HD + d) * p.vt_ld + tile.vt_col0 + tc * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
  (void)kv_dim;
}
int launch_kv_commit(const CommitParams &p, hipStream_t st) {
  if (p.n_tiles <= 0) return 0;
  dim3 grid(p.n_tiles, p.n_kv_heads);
  if (p.head_dim == 128) hipLaunchKernelGGL(kv_commit_kernel<128>, grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL(kv_commit_kernel<64>, grid, dim3(256), 0, st, p);
  return 0;
}

// -------------------------------------------------------- token scales -----
// One wave per token: absmax of its K row and of its V row (bf16 values as they will be stored),
// scale = max(absmax, 1e-12) / 448 written at the token's cache slot.
__global__ __launch_bounds__(256) void token_scale_kernel(TokenScaleParams p) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= p.T) return;
  float ak = 0.f, av = 0.f;
  for (int c = lane; c < p.kv_dim / 8; c += 64) {
    const uint4 k = *(const uint4 *)(p.k_src + (int64_t)row * p.ld_src + c * 8);
    const uint4 v = *(const uint4 *)(p.v_src + (int64_t)row * p.ld_src + c * 8);
    const uint32_t kw[4] = {k.x, k.y, k.z, k.w}, vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      ak = fmaxf(ak, fmaxf(fabsf(bf16lo(kw[e])), fabsf(bf16hi(kw[e]))));
      av = fmaxf(av, fmaxf(fabsf(bf16lo(vw[e])), fabsf(bf16hi(vw[e]))));
    }
  }
  for (int o = 32; o > 0; o >>= 1) { ak = fmaxf(ak, __shfl_xor(ak, o)); av = fmaxf(av, __shfl_xor(av, o)); }
  if (lane == 0) {
    const int64_t slot = p.slots[row];
    p.scales[slot] = fmaxf(ak, 1e-12f) / 448.0f;
    p.scales[p.n_slots + slot] = fmaxf(av, 1e-12f) / 448.0f;
  }
}
int launch_token_scales(const TokenScaleParams &p, hipStream_t st) {
  if (p.T <= 0) return 0;
  hipLaunchKernelGGL(token_scale_kernel, dim3((p.T + 3) / 4), dim3(256), 0, st, p);
  return 0;
}

// ----------------------------------------------------------- QKV finish ----
// grid (T, Hq + 2*Hkv), hd/2 threads: thread i owns the rotary pair (i, i + hd/2) of one head of one row.
__global__ void qkv_finish_kernel(QkvFinishParams p) {
  const int row = blockIdx.x, hs = blockIdx.y, i = threadIdx.x;
  const int hd = p.head_dim, half = hd / 2;
  const int kind = hs < p.n_q_heads ? 0 : (hs < p.n_q_heads + p.n_kv_heads ? 1 : 2);
  const int head = kind == 0 ? hs : (kind == 1 ? hs - p.n_q_heads : hs - p.n_q_heads - p.n_kv_heads);
  const int64_t dim = (int64_t)(kind == 0 ? p.n_q_heads : p.n_kv_heads) * hd;
  const float *src = (kind == 0 ? p.q32 : kind == 1 ? p.k32 : p.v32) + row * (p.ld32 ? (int64_t)p.ld32 : dim) + head * hd;
  bf16_t *dst = (kind == 0 ? p.q : kind == 1 ? p.k : p.v) + row * dim + head * hd;
  float x0 = src[i], x1 = src[i + half];
  if (p.n_splits > 1) {   // the K splits of the projection, added in split order
    const int64_t step = (int64_t)p.T * p.ld32;
    for (int ks = 1; ks < p.n_splits; ++ks) { x0 += src[ks * step + i]; x1 += src[ks * step + i + half]; }
  }
  if (kind != 2) {
    const float2 cs = p.cos_sin[(int64_t)row * half + i];
    const float y0 = x0 * cs.x - x1 * cs.y, y1 = x1 * cs.x + x0 * cs.y;
    x0 = y0; x1 = y1;
  }
  const bf16_t b0 = f32_to_bf16(x0), b1 = f32_to_bf16(x1);
  dst[i] = b0;
  dst[i + half] = b1;
  if (p.amax && kind != 0) {   // absmax of the values as stored (bf16-rounded)
    float a = fmaxf(fabsf(bf16_to_f32(b0)), fabsf(bf16_to_f32(b1)));
    for (int o = 32; o > 0; o >>= 1) a = fmaxf(a, __shfl_xor(a, o));
    if ((i & 63) == 0) atomicMax(p.amax + (kind == 2 ? p.n_kv_heads : 0) + head, __float_as_uint(a));
  }
}
int launch_qkv_finish(const QkvFinishParams &p, hipStream_t st) {
  if (p.T <= 0) return 0;
  hipLaunchKernelGGL(qkv_finish_kernel, dim3(p.T, p.n_q_heads + 2 * p.n_kv_heads), dim3(p.head_dim / 2), 0, st, p);
  return 0;
}

// ----------------------------------------------------------- early exit ----
// One workgroup per row: max, then sum of exp(x - max); the largest probability is 1 / that sum.
__global__ __launch_bounds__(256) void early_exit_flags_kernel(const float *early, int32_t V, float threshold, int32_t *flags) {
  __shared__ float red[4];
  const float *x = early + (int64_t)blockIdx.x * V;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float mx = -INFINITY;
  for (int i = tid; i < V; i += 256) mx = fmaxf(mx, x[i]);
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int i = tid; i < V; i += 256) sum += __expf(x[i] - mx);
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) flags[blockIdx.x] = (1.0f / (red[0] + red[1] + red[2] + red[3])) > threshold ? 1 : 0;
}
__global__ void early_exit_select_kernel(const float *early, const int32_t *flags, float *logits, int32_t V) {
  if (!flags[blockIdx.y]) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < V) logits[(int64_t)blockIdx.y * V + i] = early[(int64_t)blockIdx.y * V + i];
}
int launch_early_exit_flags(const float *early, int32_t B, int32_t V, float threshold, int32_t *flags, hipStream_t st) {
  if (B <= 0) return 0;
  hipLaunchKernelGGL(early_exit_flags_kernel, dim3(B), dim3(256), 0, st, early, V, threshold, flags);
  return 0;
}
int launch_early_exit_select(const float *early, const int32_t *flags, float *logits, int32_t B, int32_t V, hipStream_t st) {
  if (B <= 0) return 0;
  hipLaunchKernelGGL(early_exit_select_kernel, dim3((V + 255) / 256, B), dim3(256), 0, st, early, flags, logits, V);
  return 0;
}

// ----------------------------------------------------------- KV gather -----
// One workgroup per (64-position tile, KV head) of a sequence whose prompt continues over a cached
// prefix: copies the tile's K rows out of the paged cache into consecutive rows and its V rows
// into V^T columns (through LDS, as above), dequantising e4m3 codes with the layer's scales to
// the bf16 values every other reader of the cache sees.  Columns past n_valid are zero filled.
template <int HD>
__global__ __launch_bounds__(256) void kv_gather_kernel(GatherParams p) {
  constexpr int CH = HD / 8;  // 8-element chunks per row
  __shared__ bf16_t sv[64][HD + 8];
  const GatherTile tile = p.tiles[blockIdx.x];
  const int head = blockIdx.y;
  const int tid = threadIdx.x;
  const int kv_dim = p.n_kv_heads * HD;
  float sk = 1.f, svs = 1.f;
  if (p.fp8 == 1) { sk = p.scales[head]; svs = p.scales[p.n_kv_heads + head]; }
  for (int i = tid; i < 64 * CH; i += 256) {
    const int r = i / CH, c = i % CH;
    uint4 kq = make_uint4(0, 0, 0, 0), vq = make_uint4(0, 0, 0, 0);
    if (r < tile.n_valid) {
      const int pos = tile.pos0 + r;
      int blk = p.block_tables[(int64_t)tile.seq * p.max_blocks_per_seq + pos / SKV_BLOCK];
      blk = blk < 0 ? 0 : (blk >= p.n_blocks ? p.n_blocks - 1 : blk);   // bad ids were reported by the plan; stay inside the pool
      const int64_t slot = (int64_t)blk * SKV_BLOCK + pos % SKV_BLOCK;
      const int64_t src = (slot * p.n_kv_heads + head) * HD + c * 8;
      if (p.fp8 == 2) { sk = p.scales[slot]; svs = p.scales[(int64_t)p.n_blocks * SKV_BLOCK + slot]; }
      if (!p.fp8) {
        kq = *(const uint4 *)((const bf16_t *)p.cache_k + src);
        vq = *(const uint4 *)((const bf16_t *)p.cache_v + src);
      } else {
        const uint2 kc = *(const uint2 *)((const uint8_t *)p.cache_k + src);
        const uint2 vc = *(const uint2 *)((const uint8_t *)p.cache_v + src);
        const uint32_t kcw[2] = {kc.x, kc.y}, vcw[2] = {vc.x, vc.y};
        uint32_t kw[4], vw[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t k2 = kcw[e / 2] >> ((e & 1) * 16), v2 = vcw[e / 2] >> ((e & 1) * 16);
          kw[e] = pack_bf16x2(e4m3fn_to_f32((uint8_t)k2) * sk, e4m3fn_to_f32((uint8_t)(k2 >> 8)) * sk);
          vw[e] = pack_bf16x2(e4m3fn_to_f32((uint8_t)v2) * svs, e4m3fn_to_f32((uint8_t)(v2 >> 8)) * svs);
        }
        kq = make_uint4(kw[0], kw[1], kw[2], kw[3]);
        vq = make_uint4(vw[0], vw[1], vw[2], vw[3]);
      }
      *(uint4 *)(p.k_dst + (int64_t)(tile.k_row0 + r) * kv_dim + head * HD + c * 8) = kq;
    }
    const uint32_t w[4] = {vq.x, vq.y, vq.z, vq.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sv[r][c * 8 + 2 * e] = (bf16_t)(w[e] & 0xffff);
      sv[r][c * 8 + 2 * e + 1] = (bf16_t)(w[e] >> 16);
    }
  }
  __syncthreads();
  // V^T: thread writes 8 consecutive positions of one dim (16 bytes)
  for (int i = tid; i < HD * 8; i += 256) {
    const int d = i / 8, tc = i % 8;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (uint32_t)sv[tc * 8 + 2 * e][d] | ((uint32_t)sv[tc * 8 + 2 * e + 1][d] << 16);
    *(uint4 *)(p.vt + (int64_t)(head * HD + d) * p.vt_ld + tile.vt_col0 + tc * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}
int launch_kv_gather(const GatherParams &p, hipStream_t st) {
  if (p.n_tiles <= 0) return 0;
  dim3 grid(p.n_tiles, p.n_kv_heads);
  if (p.head_dim == 128) hipLaunchKernelGGL(kv_gather_kernel<128>, grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL(kv_gather_kernel<64>, grid, dim3(256), 0, st, p);
  return 0;
}

__global__ void fp8_quantize_kernel(const float *x, float scale, uint8_t *codes, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    float y = x[i] / scale;
    codes[i] = f32_to_e4m3fn(y);
  }
}
int launch_fp8_quantize(const float *x, float scale, uint8_t *codes, int64_t n, hipStream_t st) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(fp8_quantize_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, scale, codes, n);
  return 0;
}

// ------------------------------------------------- split-KV combine --------
// partial layout: [row][head][split][hd + 2] = (o[hd] unnormalised, m, l), m in log2 units.
__global__ void decode_combine_kernel(const float *partial, bf16_t *out, const DecodeRow *rows, int n_q_heads, int hd, int n_split) {
  int row = blockIdx.x, head = blockIdx.y, d = threadIdx.x;
  if (d >= hd) return;
  const int64_t out_row = rows[row].out_row;
  const float *base = partial + ((int64_t)(row * n_q_heads + head) * n_split) * (hd + 2);
  // eight splits at a time, all their loads requested before the first use (one memory latency per
  // group instead of one per split); an empty split carries m = -inf and enters with weight 0
  constexpr int G = 8;
  float m = -INFINITY;
  for (int s0 = 0; s0 < n_split; s0 += G) {
    float mv[G];
#pragma unroll
    for (int i = 0; i < G; ++i) mv[i] = s0 + i < n_split ? base[(s0 + i) * (hd + 2) + hd] : -INFINITY;
#pragma unroll
    for (int i = 0; i < G; ++i) m = fmaxf(m, mv[i]);
  }
  float acc = 0.f, l = 0.f;
  for (int s0 = 0; s0 < n_split; s0 += G) {
    float mv[G], ov[G], lv[G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const bool in = s0 + i < n_split;
      const float *ps = base + (in ? s0 + i : 0) * (hd + 2);
      mv[i] = in ? ps[hd] : -INFINITY;
      ov[i] = ps[d];
      lv[i] = ps[hd + 1];
    }
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const float w = (mv[i] == -INFINITY) ? 0.f : exp2f(mv[i] - m);
      acc += w * ov[i];
      l += w * lv[i];
    }
  }
  out[out_row * n_q_heads * hd + head * hd + d] = f32_to_bf16(acc / l);
}
int launch_decode_combine(const float *partial, bf16_t *out, const DecodeRow *rows, int32_t n_rows,
                          int32_t n_q_heads, int32_t head_dim, int32_t n_split, hipStream_t st) {
  if (n_rows <= 0) return 0;
  hipLaunchKernelGGL(decode_combine_kernel, dim3(n_rows, n_q_heads), dim3(head_dim), 0, st, partial, out, rows, n_q_heads, head_dim, n_split);
  return 0;
}
