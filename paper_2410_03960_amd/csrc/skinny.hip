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
#include "common.h"

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

  const int nsteps = (p.K + 31) / 32;
  for (int s0 = wave; s0 < nsteps; s0 += SK_WAVES * UN) {
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
      if (m < p.M) {
        if constexpr (EPI == EPI_STORE_F32) {
          *(float4 *)((float *)p.C + (int64_t)m * p.N + n) = make_float4(x[0][0], x[0][1], x[0][2], x[0][3]);
        } else {
          bf16_t *dst = (bf16_t *)p.C + (int64_t)m * p.N + n;
          float o[4] = {x[0][0], x[0][1], x[0][2], x[0][3]};
          if constexpr (EPI == EPI_RESID) {
            uint2 r = *(const uint2 *)dst;
            o[0] += bf16lo(r.x); o[1] += bf16hi(r.x); o[2] += bf16lo(r.y); o[3] += bf16hi(r.y);
          }
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

template <int MB, int NB>
int launch_mb(const SkinnyParams &p, int epi, hipStream_t st) {
  dim3 grid(p.N / (16 * NB)), block(SK_WAVES * 64);
  switch (epi) {
    case EPI_STORE_BF16: hipLaunchKernelGGL((skinny_kernel<MB, NB, EPI_STORE_BF16>), grid, block, 0, st, p); return 0;
    case EPI_STORE_F32: hipLaunchKernelGGL((skinny_kernel<MB, NB, EPI_STORE_F32>), grid, block, 0, st, p); return 0;
    case EPI_RESID: hipLaunchKernelGGL((skinny_kernel<MB, NB, EPI_RESID>), grid, block, 0, st, p); return 0;
    case EPI_SWIGLU:
      if constexpr (NB <= 2) { hipLaunchKernelGGL((skinny_kernel<MB, NB, EPI_SWIGLU>), grid, block, 0, st, p); return 0; }
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
