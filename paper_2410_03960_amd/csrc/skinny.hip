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
// partial sums and a second small kernel adds them in a fixed order and applies
// the epilogue (deterministic, unlike atomic accumulation).
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
    wrow[nb] = p.W + (int64_t)(n0 + nb * 16 + l16) * p.K + kq * 8;
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
  for (int s0 = s_begin + wave; s0 < nsteps; s0 += SK_WAVES * UN) {
    uint4 wv[UN][NJ], av[UN][MB];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + u * SK_WAVES;
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
  if (ksplit > 1) {
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
  if (p.M <= 16) return launch_mb<1, 1>(p, epi, st);
  if (p.M <= 32) return (p.N % 32 == 0) ? launch_mb<2, 2>(p, epi, st) : launch_mb<2, 1>(p, epi, st);
  if (p.M <= 48) return launch_wide<3>(p, epi, st);
  if (p.M <= 64) return launch_wide<4>(p, epi, st);
  return launch_wide<5>(p, epi, st);
}
