// Weight-streaming GEMM for the last-token tail (M <= 80 rows):
//   C[M,N] = A[M,K] * W[N,K]^T     (optionally a second weight for SwiGLU)
// HBM-bound: every weight byte is read once.  A workgroup owns 16 output
// columns; its 8 waves split K in interleaved 32-wide steps and each issues
// v_mfma_f32_16x16x32_bf16 with the weight rows as first operand, so a lane
// ends up with 4 consecutive output columns of one activation row.  The eight
// partial sums meet in LDS.
#include "common.h"

namespace {

constexpr int SK_WAVES = 8;

template <int MB, int EPI>
__global__ __launch_bounds__(SK_WAVES * 64) void skinny_kernel(SkinnyParams p) {
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  __shared__ float red[SK_WAVES][NW][64][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;
  const int n0 = blockIdx.x * 16;
  const bf16_t *wrow = p.W + (int64_t)(n0 + l16) * p.K + kq * 8;
  const bf16_t *wrow2 = (EPI == EPI_SWIGLU) ? p.W2 + (int64_t)(n0 + l16) * p.K + kq * 8 : nullptr;
  const bf16_t *arow[MB];
  bool avalid[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int m = mb * 16 + l16;
    avalid[mb] = m < p.M;
    arow[mb] = p.A + (int64_t)(avalid[mb] ? m : 0) * p.K + kq * 8;
  }
  floatx4 acc[MB][NW];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int w = 0; w < NW; ++w) acc[mb][w] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int nsteps = (p.K + 31) / 32;
  constexpr int UN = 4;
  for (int s0 = wave; s0 < nsteps; s0 += SK_WAVES * UN) {
    uint4 wv[UN], wv2[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + u * SK_WAVES;
      const int k = s * 32;
      const bool ok = (s < nsteps) && (k + kq * 8 + 8 <= p.K);
      wv[u] = ok ? *(const uint4 *)(wrow + k) : make_uint4(0, 0, 0, 0);
      if constexpr (EPI == EPI_SWIGLU) wv2[u] = ok ? *(const uint4 *)(wrow2 + k) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = s0 + u * SK_WAVES;
      const int k = s * 32;
      const bool ok = (s < nsteps) && (k + kq * 8 + 8 <= p.K);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        uint4 av = (ok && avalid[mb]) ? *(const uint4 *)(arow[mb] + k) : make_uint4(0, 0, 0, 0);
        bf16x8 af = __builtin_bit_cast(bf16x8, av);
        acc[mb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[u]), af, acc[mb][0], 0, 0, 0);
        if constexpr (EPI == EPI_SWIGLU)
          acc[mb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv2[u]), af, acc[mb][1], 0, 0, 0);
      }
    }
  }

  // acc[mb][w][v] = C[m = mb*16 + l16][n = n0 + 4*kq + v] partial over this wave's k steps
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][w][lane][v] = acc[mb][w][v];
    __syncthreads();
    if (wave == 0) {
      float x[NW][4];
#pragma unroll
      for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float sum = 0.f;
#pragma unroll
          for (int ww = 0; ww < SK_WAVES; ++ww) sum += red[ww][w][lane][v];
          x[w][v] = sum;
        }
      const int m = mb * 16 + l16, n = n0 + 4 * kq;
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
            for (int v = 0; v < 4; ++v) o[v] = x[0][v] / (1.f + __expf(-x[0][v])) * x[1][v];
          }
          *(uint2 *)dst = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
        }
      }
    }
    __syncthreads();
  }
}

template <int MB>
int launch_mb(const SkinnyParams &p, int epi, hipStream_t st) {
  dim3 grid(p.N / 16), block(SK_WAVES * 64);
  switch (epi) {
    case EPI_STORE_BF16: hipLaunchKernelGGL((skinny_kernel<MB, EPI_STORE_BF16>), grid, block, 0, st, p); return 0;
    case EPI_STORE_F32: hipLaunchKernelGGL((skinny_kernel<MB, EPI_STORE_F32>), grid, block, 0, st, p); return 0;
    case EPI_RESID: hipLaunchKernelGGL((skinny_kernel<MB, EPI_RESID>), grid, block, 0, st, p); return 0;
    case EPI_SWIGLU: hipLaunchKernelGGL((skinny_kernel<MB, EPI_SWIGLU>), grid, block, 0, st, p); return 0;
  }
  return -1;
}

}  // namespace

int launch_skinny(const SkinnyParams &p, int epi, hipStream_t st) {
  if (p.M <= 0 || p.N <= 0) return 0;
  if (p.M > 80 || (p.N % 16) != 0 || (p.K % 8) != 0) return -1;
  if (p.M <= 16) return launch_mb<1>(p, epi, st);
  if (p.M <= 32) return launch_mb<2>(p, epi, st);
  return launch_mb<5>(p, epi, st);
}
