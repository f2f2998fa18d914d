// Weight-streaming GEMM for few rows (M <= 80: the last-token tail, decode steps):
//   C[M,N] = A[M,K] * W[N,K]^T     (optionally a second weight for SwiGLU)
// HBM-bound: every weight byte is read once.  A workgroup owns 16*NB output
// columns; its 8 waves split K in interleaved 32-wide steps and each issues
// v_mfma_f32_16x16x32_bf16 with the weight rows as first operand, so a lane
// ends up with 4 consecutive output columns of one activation row per column
// block.  The eight partial sums meet in LDS.
// Every workgroup reads all of A (from L2), 16*MB rows against its 16*NB weight
// rows: with many rows the activation reads would outweigh the weights, so NB
// grows with MB (fewer, wider workgroups); with up to 16 rows NB = 1 keeps the
// most workgroups streaming.
// A CU sustains only a fraction of its share of HBM bandwidth on one such stream
// (loads in flight / latency), so every CU has to stream: when there are fewer
// column tiles than CUs, K is split over blockIdx.y, the splits write fp32
// partial sums and a second small kernel (or the consumer of the result) adds
// them in a fixed order and applies the epilogue (deterministic, unlike atomic
// accumulation).
// Three kernels: skinny_kernel (above; any K % 8 == 0, activations from L2),
// skinny_lds_kernel (K % 512 == 0, up to 32 rows: the activation slice of a
// workgroup resident in LDS) and skinny_seq_kernel (K % 512 == 0, 33..80 rows:
// slices walked in sequence behind a producer wave).
#include "common.h"

#include <algorithm>

namespace {

constexpr int SK_WAVES = 8;

template <int MB, int NB, int EPI>
__global__ __launch_bounds__(SK_WAVES * 64) void skinny_kernel(SkinnyParams p) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr int NJ = NW * NB;                       // weight-row blocks per workgroup
  constexpr int UN = NJ >= 4 ? 2 : 4;               // k steps in flight per wave
  __shared__ float red[SK_WAVES][NJ][64][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;
  const int n0 = blockIdx.x * 16 * NB;
  const bf16_t *wrow[NJ];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    wrow[nb] = (p.wtab ? p.wtab[n0 / 16 + nb] + (int64_t)l16 * p.K : p.W + (int64_t)(n0 + nb * 16 + l16) * p.K) + kq * 8;
    if constexpr (EPI == EPI_SWIGLU) wrow[NB + nb] = p.W2 + (int64_t)(n0 + nb * 16 + l16) * p.K + kq * 8;
  }
  const bf16_t *arow[MB];
  bool avalid[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int m = mb * 16 + l16;
    avalid[mb] = m < p.M;
    arow[mb] = p.A + (int64_t)(avalid[mb] ? m : 0) * p.K + kq * 8;
  }
  floatx4 acc[MB][NJ];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[mb][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // k steps of this split
  const int all_steps = (p.K + 31) / 32;
  const int per_split = (all_steps + (int)gridDim.y - 1) / (int)gridDim.y;
  const int s_begin = blockIdx.y * per_split;
  const int nsteps = (s_begin + per_split) < all_steps ? (s_begin + per_split) : all_steps;
  // (a wave takes UN consecutive steps: both 64-byte halves of a 128-byte line of a weight row are then
  // requested by the same wave back to back; with the steps dealt out one by one, two waves fetched each line)
  for (int s0 = s_begin + wave * UN; s0 < nsteps; s0 += SK_WAVES * UN) {
    uint4 wv[UN][NJ], av[UN][MB];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + u;
      const int k = s * 32;
      const bool ok = (s < nsteps) && (k + kq * 8 + 8 <= p.K);
#pragma unroll
      for (int j = 0; j < NJ; ++j) wv[u][j] = ok ? *(const uint4 *)(wrow[j] + k) : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) av[u][mb] = (ok && avalid[mb]) ? *(const uint4 *)(arow[mb] + k) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[mb][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[u][j]), __builtin_bit_cast(bf16x8, av[u][mb]), acc[mb][j], 0, 0, 0);
  }

  // acc[mb][w*NB + nb][v] = C[m = mb*16 + l16][n = n0 + nb*16 + 4*kq + v] (weight w) partial over this wave's k steps
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][j][lane][v] = acc[mb][j][v];
    __syncthreads();
    if (wave < NB) {   // wave nb finishes column block nb
      const int nb = wave;
      float x[NW][4];
#pragma unroll
      for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float sum = 0.f;
#pragma unroll
          for (int ww = 0; ww < SK_WAVES; ++ww) sum += red[ww][w * NB + nb][lane][v];
          x[w][v] = sum;
        }
      const int m = mb * 16 + l16, n = n0 + nb * 16 + 4 * kq;
      if (gridDim.y > 1) {   // partial[split][w][m][n]
        if (m < p.M) {
#pragma unroll
          for (int w = 0; w < NW; ++w)
            *(float4 *)(p.partial + (((int64_t)blockIdx.y * NW + w) * p.M + m) * p.N + n) = make_float4(x[w][0], x[w][1], x[w][2], x[w][3]);
        }
      } else if (m < p.M) {
        if constexpr (EPI == EPI_STORE_F32) {
          *(float4 *)((float *)p.C + (int64_t)m * p.N + n) = make_float4(x[0][0], x[0][1], x[0][2], x[0][3]);
        } else if constexpr (EPI == EPI_RESID) {
          float4 *dst = (float4 *)((float *)p.C + (int64_t)m * p.N + n);
          const float4 r = *dst;
          *dst = make_float4(r.x + x[0][0], r.y + x[0][1], r.z + x[0][2], r.w + x[0][3]);
        } else {
          bf16_t *dst = (bf16_t *)p.C + (int64_t)m * p.N + n;
          float o[4] = {x[0][0], x[0][1], x[0][2], x[0][3]};
          if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = x[0][v] / (1.f + __expf(-x[0][v])) * x[NW - 1][v];
          }
          *(uint2 *)dst = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
        }
      }
    }
    __syncthreads();
  }
}

// sum of the K splits in split order + epilogue, 4 columns per thread
template <int EPI>
__global__ void skinny_reduce_kernel(SkinnyParams p, int ksplit) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= (int64_t)p.M * p.N) return;
  float x[NW][4];
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int ks = 0; ks < ksplit; ++ks) {
      const float4 v = *(const float4 *)(p.partial + ((int64_t)ks * NW + w) * p.M * p.N + i);
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    x[w][0] = sum.x; x[w][1] = sum.y; x[w][2] = sum.z; x[w][3] = sum.w;
  }
  if constexpr (EPI == EPI_STORE_F32) {
    *(float4 *)((float *)p.C + i) = make_float4(x[0][0], x[0][1], x[0][2], x[0][3]);
  } else if constexpr (EPI == EPI_RESID) {
    float4 *dst = (float4 *)((float *)p.C + i);
    const float4 r = *dst;
    *dst = make_float4(r.x + x[0][0], r.y + x[0][1], r.z + x[0][2], r.w + x[0][3]);
  } else {
    bf16_t *dst = (bf16_t *)p.C + i;
    float o[4] = {x[0][0], x[0][1], x[0][2], x[0][3]};
    if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
      for (int v = 0; v < 4; ++v) o[v] = x[0][v] / (1.f + __expf(-x[0][v])) * x[NW - 1][v];
    }
    *(uint2 *)dst = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
  }
}

// ---------------------------------------------------------------------------
// The same product with the activations resident in LDS (K % 512 == 0).
// Measured on the kernel above: the activation fragments, which every wave
// fetches from L2 for every k step, take as many vector-memory requests as the
// weights and cost 20-30 % of the achieved HBM rate.  Here a workgroup owns one
// K slice; its activation slice sits in LDS in MFMA operand order (filled by
// LDS-DMA, one 1 KB fragment per request: lane (row l16, quarter kq) lands at
// 16 * lane), the waves split the output columns (16-column blocks, `nbw` in a
// row per wave) and stream their weight rows through registers two groups of
// U k steps ahead, both steps of a 128-byte line in the same wave.  No
// cross-wave reduction and no barrier after the fill.  K slices go to
// blockIdx.y and meet in skinny_reduce_kernel in a fixed order.
__device__ __forceinline__ void lds_dma16(const void *gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}

template <int MB, int EPI, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void skinny_lds_kernel(SkinnyParams p, int ks_steps, int nbw) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr int U = (NW == 1 && MB <= 2) ? 8 : 4;   // k steps (of 32) per group of loads
  extern __shared__ __align__(16) unsigned char a_lds[];   // [k step][MB][64 lanes][16 bytes]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, kq = lane >> 4;
  const int all_steps = p.K / 32;
  const int s_begin = blockIdx.y * ks_steps;
  const int steps = (all_steps - s_begin) < ks_steps ? (all_steps - s_begin) : ks_steps;   // a multiple of 2U
  const int k0 = s_begin * 32;
  const int groups = steps / U;

  const int nblocks = p.N / 16;
  const int nb0 = (blockIdx.x * WAVES + wave) * nbw;
  const int nb_end = (nb0 + nbw) < nblocks ? (nb0 + nbw) : nblocks;
  const int total = nb0 < nblocks ? (nb_end - nb0) * groups : 0;   // groups of this wave, an even number

  // weight rows of this lane: group g of column block nb covers k steps g * U ...; the groups of a wave's
  // blocks are walked in order, (l_nb, l_g) being the next one to request
  int l_nb = nb0, l_g = 0;
  auto load_group = [&](uint4 (&dst)[NW][U]) {
    const int64_t koff = k0 + l_g * (U * 32) + kq * 8, off = (int64_t)(l_nb * 16 + l16) * p.K + koff;
    const bf16_t *tsrc = p.wtab ? p.wtab[l_nb] + ((int64_t)l16 * p.K + koff) : nullptr;   // (one weight, never SwiGLU)
    if (++l_g == groups) { l_g = 0; ++l_nb; }
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const bf16_t *src = tsrc ? tsrc : (w ? p.W2 : p.W) + off;
#pragma unroll
      for (int u = 0; u < U; ++u) dst[w][u] = *(const uint4 *)(src + u * 32);
    }
  };
  uint4 wa[NW][U], wb[NW][U];
  if (total > 0) load_group(wa);   // on its way while the activations arrive

  // activation slice -> LDS: fragment (k step s, row block mb) at (s * MB + mb) * 1024; rows past M repeat row M-1
  {
    typedef __attribute__((address_space(3))) void *lds_ptr_t;
    const unsigned lds_base = (unsigned)(size_t)(lds_ptr_t)a_lds;
    for (int f = wave; f < steps * MB; f += WAVES) {
      const int s = f / MB, mb = f % MB;
      int m = mb * 16 + l16;
      m = m < p.M ? m : p.M - 1;
      lds_dma16(p.A + ((int64_t)m * p.K + k0 + s * 32 + kq * 8), lds_base + f * 1024);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
  }
  if (total == 0) return;

  floatx4 acc[NW][MB];
#pragma unroll
  for (int w = 0; w < NW; ++w)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[w][mb] = floatx4{0.f, 0.f, 0.f, 0.f};
  auto compute_group = [&](const uint4 (&src)[NW][U], int g) {
    const unsigned char *fr = a_lds + (size_t)(g * U) * (MB * 1024) + lane * 16;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      bf16x8 a[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) a[mb] = *(const bf16x8 *)(fr + (u * MB + mb) * 1024);
#pragma unroll
      for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          acc[w][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, src[w][u]), a[mb], acc[w][mb], 0, 0, 0);
    }
  };
  // acc[w][mb][v] = C[m = mb*16 + l16][n = nb*16 + 4*kq + v] (weight w), over this K slice
  auto flush = [&](int nb) {
    const int n = nb * 16 + 4 * kq;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int m = mb * 16 + l16;
      if (m < p.M) {
        if (gridDim.y > 1) {   // partial[split][w][m][n]
#pragma unroll
          for (int w = 0; w < NW; ++w)
            *(float4 *)(p.partial + (((int64_t)blockIdx.y * NW + w) * p.M + m) * p.N + n) =
                make_float4(acc[w][mb][0], acc[w][mb][1], acc[w][mb][2], acc[w][mb][3]);
        } else if constexpr (EPI == EPI_STORE_F32) {
          *(float4 *)((float *)p.C + (int64_t)m * p.N + n) = make_float4(acc[0][mb][0], acc[0][mb][1], acc[0][mb][2], acc[0][mb][3]);
        } else if constexpr (EPI == EPI_RESID) {
          float4 *dst = (float4 *)((float *)p.C + (int64_t)m * p.N + n);
          const float4 r = *dst;
          *dst = make_float4(r.x + acc[0][mb][0], r.y + acc[0][mb][1], r.z + acc[0][mb][2], r.w + acc[0][mb][3]);
        } else {
          float o[4] = {acc[0][mb][0], acc[0][mb][1], acc[0][mb][2], acc[0][mb][3]};
          if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = o[v] / (1.f + __expf(-o[v])) * acc[NW - 1][mb][v];
          }
          *(uint2 *)((bf16_t *)p.C + (int64_t)m * p.N + n) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
        }
      }
#pragma unroll
      for (int w = 0; w < NW; ++w) acc[w][mb] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  };
  // two groups per iteration, one register set in flight while the other is consumed; `groups` is even, so
  // a block ends after the second group of an iteration
  int c_nb = nb0, c_g = 0;
  for (int idx = 0; idx < total; idx += 2) {
    load_group(wb);
    compute_group(wa, c_g);
    if (idx + 2 < total) load_group(wa);
    compute_group(wb, c_g + 1);
    c_g += 2;
    if (c_g == groups) { flush(c_nb); ++c_nb; c_g = 0; }
  }
}

// ---------------------------------------------------------------------------
// The LDS-resident form for many rows (M > 32), where a K slice that fits LDS is
// short (512 columns at 64 rows) and one slice per workgroup would mean many K
// splits, i.e. fp32 partial sums of 12-25 % of the weight bytes.  Here a workgroup
// walks several slices of its K range one after the other: the activation slice
// is double-buffered in LDS and filled by a producer wave of its own (LDS-DMA,
// then a wait for everything it requested, then the workgroup barrier), so the
// consumer waves never wait for an LDS-DMA request and their weight stream runs
// on across slice boundaries; a consumer keeps the accumulators of its NBW column
// blocks in registers over the whole K range.  One barrier per slice.
template <int MB, int EPI, int WAVES, int NBW>
__global__ __launch_bounds__((WAVES + 1) * 64) void skinny_seq_kernel(SkinnyParams p, int ks_steps, int n_slices) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  constexpr int U = (NBW * NW >= 4) ? 2 : 4;                                      // k steps (of 32) per group of loads
  extern __shared__ __align__(16) unsigned char a_lds[];   // [2][k step][MB][64 lanes][16 bytes]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, kq = lane >> 4;
  const int all_slices = p.K / (32 * ks_steps);
  const int sl_begin = blockIdx.y * n_slices;
  const int my_slices = (all_slices - sl_begin) < n_slices ? (all_slices - sl_begin) : n_slices;   // >= 1 by the grid
  const int k0 = sl_begin * ks_steps * 32;
  const int buf_bytes = ks_steps * MB * 1024;

  if (wave == WAVES) {
    // producer: slice s -> buffer s & 1, fragment (k step j, row block mb) at (j * MB + mb) * 1024; rows past M repeat row M-1
    typedef __attribute__((address_space(3))) void *lds_ptr_t;
    const unsigned lds_base = (unsigned)(size_t)(lds_ptr_t)a_lds;
    for (int s = 0; s <= my_slices; ++s) {
      if (s < my_slices) {
        for (int f = 0; f < ks_steps * MB; ++f) {
          const int j = f / MB, mb = f % MB;
          int m = mb * 16 + l16;
          m = m < p.M ? m : p.M - 1;
          lds_dma16(p.A + ((int64_t)m * p.K + k0 + (s * ks_steps + j) * 32 + kq * 8), lds_base + (s & 1) * buf_bytes + f * 1024);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the slice is in LDS
      }
      __builtin_amdgcn_s_barrier();           // slice s is ready / the consumers have left slice s - 1
    }
    return;
  }

  const int nblocks = p.N / 16;
  const int gps = ks_steps / U;                                       // groups per slice, even
  const int nb0 = (blockIdx.x * WAVES + wave) * NBW;
  const int total = my_slices * gps;                                  // groups of this wave
  // weight rows of this lane: a group is U k steps of all NBW column blocks (an activation fragment read from
  // LDS then feeds NBW * NW products); groups are requested in the order they are consumed.
  // (a column block past N re-reads the last one; its results are dropped)
  int64_t woff[NBW];
  const bf16_t *wt[NBW];
#pragma unroll
  for (int b = 0; b < NBW; ++b) {
    int nb = nb0 + b;
    nb = nb < nblocks ? nb : nblocks - 1;
    woff[b] = (int64_t)(nb * 16 + l16) * p.K + k0 + kq * 8;
    wt[b] = p.wtab ? p.wtab[nb] + ((int64_t)l16 * p.K + k0 + kq * 8) : nullptr;   // (one weight, never SwiGLU)
  }
  int l_idx = 0;
  auto load_group = [&](uint4 (&dst)[NBW][NW][U]) {
    const int koff = l_idx * (U * 32);
    ++l_idx;
#pragma unroll
    for (int b = 0; b < NBW; ++b)
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const bf16_t *src = (wt[b] ? wt[b] : (w ? p.W2 : p.W) + woff[b]) + koff;
#pragma unroll
        for (int u = 0; u < U; ++u) dst[b][w][u] = *(const uint4 *)(src + u * 32);
      }
  };
  uint4 wa[NBW][NW][U], wb[NBW][NW][U];
  load_group(wa);   // on its way while the first slice arrives

  floatx4 acc[NBW][NW][MB];
#pragma unroll
  for (int b = 0; b < NBW; ++b)
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) acc[b][w][mb] = floatx4{0.f, 0.f, 0.f, 0.f};

  int idx = 0;
  __builtin_amdgcn_s_barrier();   // slice 0 is in LDS
  for (int s = 0; s < my_slices; ++s) {
    const unsigned char *buf = a_lds + (s & 1) * buf_bytes + lane * 16;
    for (int g = 0; g < gps; g += 2) {
      load_group(wb);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const unsigned char *fr = buf + (size_t)((g + half) * U) * (MB * 1024);
        if (half == 1 && idx + 2 < total) load_group(wa);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          bf16x8 a[MB];
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) a[mb] = *(const bf16x8 *)(fr + (u * MB + mb) * 1024);
#pragma unroll
          for (int b = 0; b < NBW; ++b)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
              for (int mb = 0; mb < MB; ++mb)
                acc[b][w][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, half ? wb[b][w][u] : wa[b][w][u]), a[mb], acc[b][w][mb], 0, 0, 0);
        }
      }
      idx += 2;
    }
    // every LDS read of this slice has returned (its values went into the products above); no wait for the
    // weight loads in flight
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  }

  // acc[b][w][mb][v] = C[m = mb*16 + l16][n = (nb0 + b)*16 + 4*kq + v] (weight w), over this K range
#pragma unroll
  for (int b = 0; b < NBW; ++b) {
    const int nb = nb0 + b;
    if (nb >= nblocks) continue;
    const int n = nb * 16 + 4 * kq;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int m = mb * 16 + l16;
      if (m >= p.M) continue;
      if (gridDim.y > 1) {   // partial[split][w][m][n]
#pragma unroll
        for (int w = 0; w < NW; ++w)
          *(float4 *)(p.partial + (((int64_t)blockIdx.y * NW + w) * p.M + m) * p.N + n) =
              make_float4(acc[b][w][mb][0], acc[b][w][mb][1], acc[b][w][mb][2], acc[b][w][mb][3]);
      } else if constexpr (EPI == EPI_STORE_F32) {
        *(float4 *)((float *)p.C + (int64_t)m * p.N + n) = make_float4(acc[b][0][mb][0], acc[b][0][mb][1], acc[b][0][mb][2], acc[b][0][mb][3]);
      } else if constexpr (EPI == EPI_RESID) {
        float4 *dst = (float4 *)((float *)p.C + (int64_t)m * p.N + n);
        const float4 r = *dst;
        *dst = make_float4(r.x + acc[b][0][mb][0], r.y + acc[b][0][mb][1], r.z + acc[b][0][mb][2], r.w + acc[b][0][mb][3]);
      } else {
        float o[4] = {acc[b][0][mb][0], acc[b][0][mb][1], acc[b][0][mb][2], acc[b][0][mb][3]};
        if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
          for (int v = 0; v < 4; ++v) o[v] = o[v] / (1.f + __expf(-o[v])) * acc[b][NW - 1][mb][v];
        }
        *(uint2 *)((bf16_t *)p.C + (int64_t)m * p.N + n) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
      }
    }
  }
}

struct SeqPlan {
  bool ok;
  int waves, nbw, ks_steps, n_slices, ksplit;
  size_t lds_bytes, partial_bytes;
};
// Shape of the launch for M > 32: column blocks per workgroup (waves x nbw) and K ranges, chosen by the
// bytes that move besides the weights -- every workgroup fetches the activation rows of its K range from
// L2 (n_cg * M * K * 2 bytes in total over n_cg column groups, whatever the K split), K splits write and
// re-read fp32 partial sums (2 * ksplit * nw * M * N * 4 bytes) and, for the epilogues that cannot leave
// the sum to their consumer, need a second launch -- scaled by how evenly the workgroups fill the 256 CUs
// (one workgroup per CU: the two activation buffers take most of LDS).  Measured at 64 rows (us per call,
// previous one-slice form -> this one): 128256 x 4096 296 -> 196, 28672 x 4096 64.4 -> 61.2 and no second
// launch, 4096 x 4096 18.0 -> 16.5, 4096 x 14336 36.8 -> 36.8; at 80 rows 28672 x 4096 97.7 -> 67.1.
SeqPlan plan_seq(int M, int N, int K, int nw, bool consumer_sums, size_t partial_cap) {
  SeqPlan best{};
  if (M <= 32 || M > 80 || (N % 16) != 0 || (K % 512) != 0) return best;
  const int MB = (M + 15) / 16;
  const int ks_steps = MB <= 4 ? 16 : 8;                      // 2 x 48-64 KB, 2 x 40 KB of LDS
  const int all_slices = K / (32 * ks_steps), nblocks = N / 16;
  const double w_bytes = 2.0 * nw * N * K;
  double best_cost = 0;
  for (int waves = 4; waves <= 8; waves += 4)
    for (int nbw = 1; nbw <= 4; nbw *= 2) {
      if (nw == 2 && nbw * waves > 8) continue;               // (two weights: register budget of the instantiations below)
      const int n_cg = (nblocks + waves * nbw - 1) / (waves * nbw);
      for (int want = 1; want <= std::min(SKINNY_MAX_SPLIT, all_slices); ++want) {
        const int n_slices = (all_slices + want - 1) / want;
        const int ksplit = (all_slices + n_slices - 1) / n_slices;
        if (ksplit != want) continue;
        const int64_t wgs = (int64_t)n_cg * ksplit;
        const size_t partial = ksplit > 1 ? (size_t)ksplit * nw * M * N * 4 : 0;
        if (partial > partial_cap) continue;
        const double a_bytes = 0.75 * (double)n_cg * M * K * 2, p_bytes = 2.0 * partial;   // (L2 hits: cheaper than the partial sums' trip to memory)
        const double second = (ksplit > 1 && !consumer_sums) ? 25e6 : 0;   // a launch, in bytes at the streaming rate
        const int64_t n_rounds = (wgs + 255) / 256;   // every further round pays its own fill and uneven end
        const double rounds = (double)n_rounds * 256.0 / (double)wgs * (1.0 + 0.15 * (double)(n_rounds - 1));
        const double cost = (w_bytes + a_bytes + p_bytes + second) * rounds;
        if (!best.ok || cost < best_cost) {
          best_cost = cost;
          best = SeqPlan{true, waves, nbw, ks_steps, n_slices, ksplit, (size_t)2 * ks_steps * MB * 1024, partial};
        }
      }
    }
  return best;
}
template <int MB, int EPI, int WAVES, int NBW>
int launch_seq_k(const SkinnyParams &p, const SeqPlan &pl, hipStream_t st) {
  auto kern = skinny_seq_kernel<MB, EPI, WAVES, NBW>;
  static bool attr = false;
  if (!attr) {
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes) != hipSuccess) return -1;
    attr = true;   // (the size depends on MB only)
  }
  const int nblocks = p.N / 16;
  dim3 grid((nblocks + WAVES * NBW - 1) / (WAVES * NBW), pl.ksplit);
  hipLaunchKernelGGL(kern, grid, dim3((WAVES + 1) * 64), pl.lds_bytes, st, p, pl.ks_steps, pl.n_slices);
  if (pl.ksplit > 1 && p.n_splits_out) *p.n_splits_out = pl.ksplit;   // the consumer adds the splits
  else if (pl.ksplit > 1) {
    const int64_t quads = (int64_t)p.M * p.N / 4;
    hipLaunchKernelGGL((skinny_reduce_kernel<EPI>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p, pl.ksplit);
  }
  return 0;
}
template <int MB, int EPI>
int launch_seq_e(const SkinnyParams &p, const SeqPlan &pl, hipStream_t st) {
  if constexpr (EPI != EPI_SWIGLU) {
    if (pl.nbw == 4) return pl.waves == 4 ? launch_seq_k<MB, EPI, 4, 4>(p, pl, st) : launch_seq_k<MB, EPI, 8, 4>(p, pl, st);
    if (pl.waves == 8 && pl.nbw == 2) return launch_seq_k<MB, EPI, 8, 2>(p, pl, st);
  }
  if (pl.waves == 8 && pl.nbw == 1) return launch_seq_k<MB, EPI, 8, 1>(p, pl, st);
  if (pl.waves == 4 && pl.nbw == 2) return launch_seq_k<MB, EPI, 4, 2>(p, pl, st);
  if (pl.waves == 4 && pl.nbw == 1) return launch_seq_k<MB, EPI, 4, 1>(p, pl, st);
  return -1;
}
template <int MB>
int launch_seq_m(const SkinnyParams &p, int epi, const SeqPlan &pl, hipStream_t st) {
  switch (epi) {
    case EPI_STORE_BF16: return launch_seq_e<MB, EPI_STORE_BF16>(p, pl, st);
    case EPI_STORE_F32: return launch_seq_e<MB, EPI_STORE_F32>(p, pl, st);
    case EPI_RESID: return launch_seq_e<MB, EPI_RESID>(p, pl, st);
    case EPI_SWIGLU: return launch_seq_e<MB, EPI_SWIGLU>(p, pl, st);
  }
  return -1;
}
int launch_seq(const SkinnyParams &p, int epi, const SeqPlan &pl, hipStream_t st) {
  switch ((p.M + 15) / 16) {
    case 3: return launch_seq_m<3>(p, epi, pl, st);
    case 4: return launch_seq_m<4>(p, epi, pl, st);
    default: return launch_seq_m<5>(p, epi, pl, st);
  }
}

struct LdsPlan {
  bool ok;
  int waves, ks_steps, ksplit, nbw;
  size_t lds_bytes, partial_bytes;
};
// How the one-slice LDS-resident form would run this shape (M <= 32); ok = false: it cannot, or the first
// kernel does better (few column blocks: its workgroups split K among their waves and need no second
// pass).  Measured on the 8B shapes with 8 rows: slices of 2048 (up to 16 rows) / 1024 columns of K, two
// column blocks in a row per wave when there are many.
LdsPlan plan_lds(int M, int N, int K, int nw, size_t partial_cap) {
  LdsPlan pl{};
  if (M < 1 || M > 32 || (N % 16) != 0 || (K % 512) != 0) return pl;
  const int MB = (M + 15) / 16;
  const int U = (nw == 1) ? 8 : 4;
  const int all_steps = K / 32, nblocks = N / 16;
  const int steps_cap = MB == 1 ? 64 : 32;                          // 64 KB of LDS
  int ksplit = (all_steps + steps_cap - 1) / steps_cap;
  const int ks_steps = ((all_steps + ksplit - 1) / ksplit + 2 * U - 1) / (2 * U) * (2 * U);
  ksplit = (all_steps + ks_steps - 1) / ks_steps;
  pl.ks_steps = ks_steps; pl.ksplit = ksplit;
  const int64_t streams = (int64_t)nblocks * ksplit;                // (column block, K slice) pairs; a wave takes nbw of them in a row
  if (streams < 1024) return pl;                                    // too few: the first kernel keeps more CUs busy
  pl.nbw = streams >= 3200 ? 2 : 1;
  pl.waves = 8;
  pl.lds_bytes = (size_t)ks_steps * MB * 1024;
  pl.partial_bytes = ksplit > 1 ? (size_t)ksplit * nw * M * N * 4 : 0;
  pl.ok = pl.partial_bytes <= partial_cap && pl.lds_bytes <= 160 * 1024;
  return pl;
}

template <int MB, int EPI, int WAVES>
int launch_lds_w(const SkinnyParams &p, const LdsPlan &pl, hipStream_t st) {
  auto kern = skinny_lds_kernel<MB, EPI, WAVES>;
  static size_t attr = 0;
  if (pl.lds_bytes > attr) {
    if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes) != hipSuccess) return -1;
    attr = pl.lds_bytes;
  }
  const int nblocks = p.N / 16;
  dim3 grid((nblocks + WAVES * pl.nbw - 1) / (WAVES * pl.nbw), pl.ksplit);
  hipLaunchKernelGGL(kern, grid, dim3(WAVES * 64), pl.lds_bytes, st, p, pl.ks_steps, pl.nbw);
  if (pl.ksplit > 1 && p.n_splits_out) *p.n_splits_out = pl.ksplit;   // the consumer adds the splits
  else if (pl.ksplit > 1) {
    const int64_t quads = (int64_t)p.M * p.N / 4;
    hipLaunchKernelGGL((skinny_reduce_kernel<EPI>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p, pl.ksplit);
  }
  return 0;
}
template <int MB>
int launch_lds_m(const SkinnyParams &p, int epi, const LdsPlan &pl, hipStream_t st) {
  switch (epi) {
    case EPI_STORE_BF16: return launch_lds_w<MB, EPI_STORE_BF16, 8>(p, pl, st);
    case EPI_STORE_F32: return launch_lds_w<MB, EPI_STORE_F32, 8>(p, pl, st);
    case EPI_RESID: return launch_lds_w<MB, EPI_RESID, 8>(p, pl, st);
    case EPI_SWIGLU: return launch_lds_w<MB, EPI_SWIGLU, 8>(p, pl, st);
  }
  return -1;
}
int launch_lds(const SkinnyParams &p, int epi, const LdsPlan &pl, hipStream_t st) {
  return p.M <= 16 ? launch_lds_m<1>(p, epi, pl, st) : launch_lds_m<2>(p, epi, pl, st);
}

template <int MB, int NB, int EPI>
int launch_kernels(const SkinnyParams &p, hipStream_t st) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  const int tiles = p.N / (16 * NB);
  // split K while the column tiles leave CUs idle: up to 4 splits, each at least 16 k steps per wave pass
  int ksplit = 1;
  if (p.partial && MB >= 3 && tiles < 256) {
    ksplit = std::min(SKINNY_MAX_SPLIT, 256 / tiles);
    ksplit = std::min(ksplit, std::max(1, p.K / (32 * SK_WAVES * 4)));
    if ((size_t)ksplit * NW * p.M * p.N * 4 > p.partial_bytes) ksplit = 1;
  }
  dim3 grid(tiles, ksplit), block(SK_WAVES * 64);
  hipLaunchKernelGGL((skinny_kernel<MB, NB, EPI>), grid, block, 0, st, p);
  if (ksplit > 1 && p.n_splits_out) *p.n_splits_out = ksplit;   // the consumer adds the splits
  else if (ksplit > 1) {
    const int64_t quads = (int64_t)p.M * p.N / 4;
    hipLaunchKernelGGL((skinny_reduce_kernel<EPI>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p, ksplit);
  }
  return 0;
}

template <int MB, int NB>
int launch_mb(const SkinnyParams &p, int epi, hipStream_t st) {
  switch (epi) {
    case EPI_STORE_BF16: return launch_kernels<MB, NB, EPI_STORE_BF16>(p, st);
    case EPI_STORE_F32: return launch_kernels<MB, NB, EPI_STORE_F32>(p, st);
    case EPI_RESID: return launch_kernels<MB, NB, EPI_RESID>(p, st);
    case EPI_SWIGLU:
      if constexpr (NB <= 2) return launch_kernels<MB, NB, EPI_SWIGLU>(p, st);
      break;
  }
  return -1;
}

template <int MB>
int launch_wide(const SkinnyParams &p, int epi, hipStream_t st) {
  // two weight matrices count double: at most four weight-row blocks per workgroup
  const int want = epi == EPI_SWIGLU ? 2 : 4;
  if (want == 4 && p.N % 64 == 0) return launch_mb<MB, 4>(p, epi, st);
  if (p.N % 32 == 0) return launch_mb<MB, 2>(p, epi, st);
  return launch_mb<MB, 1>(p, epi, st);
}

}  // namespace

int launch_skinny(const SkinnyParams &p, int epi, hipStream_t st) {
  if (p.M <= 0 || p.N <= 0) return 0;
  if (p.M > 80 || (p.N % 16) != 0 || (p.K % 8) != 0) return -1;
  if (p.n_splits_out) {
    if (epi != EPI_STORE_F32 && epi != EPI_RESID) return -1;
    *p.n_splits_out = 1;
  }
  {
    const SeqPlan sq = plan_seq(p.M, p.N, p.K, epi == EPI_SWIGLU ? 2 : 1, p.n_splits_out != nullptr, p.partial ? p.partial_bytes : 0);
    if (sq.ok) return launch_seq(p, epi, sq, st);
  }
  {
    const LdsPlan pl = plan_lds(p.M, p.N, p.K, epi == EPI_SWIGLU ? 2 : 1, p.partial ? p.partial_bytes : 0);
    if (pl.ok) return launch_lds(p, epi, pl, st);
  }
  if (p.M <= 16) return launch_mb<1, 1>(p, epi, st);
  if (p.M <= 32) return (p.N % 32 == 0) ? launch_mb<2, 2>(p, epi, st) : launch_mb<2, 1>(p, epi, st);
  if (p.M <= 48) return launch_wide<3>(p, epi, st);
  if (p.M <= 64) return launch_wide<4>(p, epi, st);
  return launch_wide<5>(p, epi, st);
}
