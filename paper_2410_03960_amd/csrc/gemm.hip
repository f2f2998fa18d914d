// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T  with fused epilogues
// (fp32 residual add, SwiGLU, 1/rms row scale + RoPE + q/k/v split, 1/rms + RoPE
// + paged KV scatter).
//
// Layout of the computation.  A workgroup owns a BM x BN tile of C and walks K
// in steps of 64.  Global -> registers -> LDS double buffering (one barrier per
// step); LDS rows are 128 bytes with the 16-byte chunk index XOR-ed by
// ((row >> 1) & 7): the LDS serves 16 lanes (256 bytes, 64 banks) per cycle, and
// with this key 16 consecutive rows of one logical chunk fall into 16 different
// 16-byte bank groups, so the MFMA operand loads (and the 16-byte stores) are
// conflict free.
// Each wave owns a WTM x 128 sub-tile and issues v_mfma_f32_32x32x16_bf16 with
// the weight rows as the first operand and the activation rows as the second,
// so an accumulator register quad holds four consecutive output columns of one
// token row: stores are 8 bytes per lane, and the RoPE partner column (n +
// head_dim/2) sits in the same lane.
//
// The weight operand is addressed through a table of row-block pointers (16
// rows each), which lets [W_Q;W_K;W_V], the 16-row interleave of W_gate/W_up and
// the concatenated [W_K;W_V] of all AcrossKV group leaders be consumed in place.
#include "common.h"
#include <type_traits>

namespace {

constexpr int BK = 64;

// Shared epilogue.  acc[bn][bm][4*jg + e] is C[m][n + e] with
// m = m_base + bm*32 + (lane & 31), n = n_base + bn*32 + 8*jg + 4*(lane >> 5).
template <int EPI, int FM, int FN>
__device__ __forceinline__ void gemm_epilogue(const GemmParams &p, floatx16 (&acc)[FN][FM], const int m_base,
                                              const int n_base, const int lane) {
  const int l32 = lane & 31, g = lane >> 5;
  // ------------------------------------------------------------ epilogue ----
  // acc[bn][bm][4*jg + e] is C[m][n + e], m = m_base + bm*32 + l32,
  // n = n_base + bn*32 + 8*jg + 4*g.

  if constexpr (EPI == EPI_STORE_BF16 || EPI == EPI_STORE_F32 || EPI == EPI_RESID) {
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      const int m = m_base + bm * 32 + l32;
      if (m >= p.M) continue;
#pragma unroll
      for (int bn = 0; bn < FN; ++bn)
#pragma unroll
        for (int jg = 0; jg < 4; ++jg) {
          const int n = n_base + bn * 32 + 8 * jg + 4 * g;
          if (n >= p.N) continue;
          float x0 = acc[bn][bm][4 * jg], x1 = acc[bn][bm][4 * jg + 1], x2 = acc[bn][bm][4 * jg + 2], x3 = acc[bn][bm][4 * jg + 3];
          if constexpr (EPI == EPI_STORE_F32) {
            *(float4 *)((float *)p.C + (int64_t)m * p.ldc + n) = make_float4(x0, x1, x2, x3);
          } else if constexpr (EPI == EPI_RESID) {
            float4 *dst = (float4 *)((float *)p.C + (int64_t)m * p.ldc + n);
            const float4 r = *dst;
            *dst = make_float4(r.x + x0, r.y + x1, r.z + x2, r.w + x3);
          } else {
            bf16_t *dst = (bf16_t *)p.C + (int64_t)m * p.ldc + n;
            *(uint2 *)dst = make_uint2(pack_bf16x2(x0, x1), pack_bf16x2(x2, x3));
          }
        }
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
    // every 32 virtual rows = 16 gate rows then the matching 16 up rows
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      const int m = m_base + bm * 32 + l32;
      if (m >= p.M) continue;
      const float rs = p.rstd ? p.rstd[m] : 1.f;
#pragma unroll
      for (int bn = 0; bn < FN; ++bn) {
        const int nv = n_base + bn * 32;
        if (nv >= p.N) continue;
#pragma unroll
        for (int jg = 0; jg < 2; ++jg) {
          const int col = nv / 2 + 8 * jg + 4 * g;
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float gt = acc[bn][bm][4 * jg + e] * rs, up = acc[bn][bm][4 * (jg + 2) + e] * rs;
            o[e] = gt * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * up;   // silu(gate) * up
          }
          *(uint2 *)((bf16_t *)p.C + (int64_t)m * p.ldc + col) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
        }
      }
    }
  } else {  // EPI_QKV / EPI_KV
    if (n_base >= p.N) return;
    const int hd = p.head_dim;
    const int half_blocks = hd / 64;          // 32-column blocks per rotary half: 2 (hd 128) or 1 (hd 64)
    const int heads_per_tile = 128 / hd;      // 1 or 2
    // classify this wave's 128 columns (uniform over the wave)
    int kind, col0, proj = 0;                 // kind 0 = q, 1 = k, 2 = v
    if constexpr (EPI == EPI_QKV) {
      if (n_base < p.q_dim) { kind = 0; col0 = n_base; }
      else if (n_base < p.q_dim + p.kv_dim) { kind = 1; col0 = n_base - p.q_dim; }
      else { kind = 2; col0 = n_base - p.q_dim - p.kv_dim; }
    } else {
      proj = n_base / (2 * p.kv_dim);
      int within = n_base % (2 * p.kv_dim);
      kind = within < p.kv_dim ? 1 : 2;
      col0 = within % p.kv_dim;
    }
    float amax_h[2] = {0.f, 0.f};
    // destination of this wave's columns, selected once (uniform over the wave): base pointer and row
    // stride in elements; rows of the paged cache go through p.slots
    bf16_t *obase;
    int64_t ostride;
    bool paged = false;
    if constexpr (EPI == EPI_QKV) {
      obase = p.q_out; ostride = p.q_dim;
      if (kind == 1) { obase = p.k_out; ostride = p.kv_dim; }
      if (kind == 2) { obase = p.v_out; ostride = p.kv_dim; }
      obase += col0;
    } else {
      obase = p.stage + n_base; ostride = p.N;
      if (!p.stage) {
        obase = p.cache + (int64_t)(p.first_cache_layer + proj) * p.cache_layer_stride + (kind == 2 ? p.cache_kv_stride : 0) + col0;
        ostride = p.kv_dim; paged = true;
      }
    }
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      const int m = m_base + bm * 32 + l32;
      const bool mv = m < p.M;
      const int mc = mv ? m : p.M - 1;
      const float rs = p.rstd ? p.rstd[mc] : 1.f;
#pragma unroll
      for (int bn = 0; bn < FN; ++bn)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[bn][bm][v] *= rs;
      if (kind != 2) {
        const float2 *cs = p.cos_sin + (int64_t)mc * (hd / 2);
        for (int hh = 0; hh < heads_per_tile; ++hh)
          for (int hb = 0; hb < half_blocks; ++hb) {
            const int blo = hh * (hd / 32) + hb, bhi = blo + half_blocks;
#pragma unroll
            for (int jg = 0; jg < 4; ++jg) {
              const int i0 = hb * 32 + 8 * jg + 4 * g;
              const float4 c01 = *(const float4 *)(cs + i0), c23 = *(const float4 *)(cs + i0 + 2);
              const float cv[4] = {c01.x, c01.z, c23.x, c23.z}, sv[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                // FN == 4: blo, bhi in 0..3; select without dynamic register indexing
                float x1 = 0.f, x2 = 0.f;
#pragma unroll
                for (int b = 0; b < FN; ++b) {
                  if (b == blo) x1 = acc[b][bm][4 * jg + e];
                  if (b == bhi) x2 = acc[b][bm][4 * jg + e];
                }
                const float y1 = x1 * cv[e] - x2 * sv[e], y2 = x2 * cv[e] + x1 * sv[e];
#pragma unroll
                for (int b = 0; b < FN; ++b) {
                  if (b == blo) acc[b][bm][4 * jg + e] = y1;
                  if (b == bhi) acc[b][bm][4 * jg + e] = y2;
                }
              }
            }
          }
      }
      // destination row pointer for this token
      int64_t orow = mc;
      if constexpr (EPI == EPI_KV) { if (paged) orow = p.slots[mc]; }
      bf16_t *dst = obase + orow * ostride;
#pragma unroll
      for (int bn = 0; bn < FN; ++bn)
#pragma unroll
        for (int jg = 0; jg < 4; ++jg) {
          float x0 = acc[bn][bm][4 * jg], x1 = acc[bn][bm][4 * jg + 1], x2 = acc[bn][bm][4 * jg + 2], x3 = acc[bn][bm][4 * jg + 3];
          const uint2 pk = make_uint2(pack_bf16x2(x0, x1), pack_bf16x2(x2, x3));
          if (mv) {
            *(uint2 *)(dst + bn * 32 + 8 * jg + 4 * g) = pk;
            if (p.amax && kind != 0) {  // absmax of the values as stored (bf16-rounded)
              float a = fmaxf(fmaxf(fabsf(bf16lo(pk.x)), fabsf(bf16hi(pk.x))), fmaxf(fabsf(bf16lo(pk.y)), fabsf(bf16hi(pk.y))));
              const int hsel = (bn * 32) / hd;  // head inside the tile (0 or 1)
              if (hsel == 0) amax_h[0] = fmaxf(amax_h[0], a); else amax_h[1] = fmaxf(amax_h[1], a);
            }
          }
        }
    }
    if (p.amax && kind != 0) {
      const int n_kv_heads = p.kv_dim / hd;
      for (int hh = 0; hh < heads_per_tile; ++hh) {
        float a = wave_max(amax_h[hh]);
        if (lane == 0) {
          int head = col0 / hd + hh;
          int c = p.first_cache_layer + proj;
          atomicMax(p.amax + ((int64_t)c * 2 + (kind == 2 ? 1 : 0)) * n_kv_heads + head, __float_as_uint(a));
        }
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_kernel(GemmParams p) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  static_assert(WTN == 128, "wave tile must span 128 output columns");
  static_assert(WTM % 32 == 0, "wave tile rows");
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int A_IT = BM * 8 / NT, B_IT = BN * 8 / NT;
  constexpr int ROWS_PER_IT = NT / 8;
  constexpr int STAGE_BYTES = (BM + BN) * 128;

  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, g = lane >> 5;

  // ---- tile assignment: consecutive tiles of a group land on one XCD ----
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= total) return;
  constexpr int GM = 8;
  const int group = logical / (GM * tiles_n);
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_group = logical % (GM * tiles_n);
  const int tm = first_m + in_group % gsz, tn = in_group / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- per-thread global load addresses ----
  const int lc = tid & 7;        // 16-byte chunk inside the 64-wide k step
  const int lr = tid >> 3;       // first row this thread loads
  const bf16_t *a_ptr[A_IT];
  const bf16_t *w_ptr[B_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    int m = m0 + lr + i * ROWS_PER_IT;
    m = m < p.M ? m : p.M - 1;
    a_ptr[i] = p.A + (int64_t)m * p.lda + lc * 8;
  }
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    int n = n0 + lr + i * ROWS_PER_IT;
    n = n < p.N ? n : p.N - 1;
    w_ptr[i] = (p.wtab ? p.wtab[n >> 4] + (int64_t)(n & 15) * p.ldw : p.W + (int64_t)n * p.ldw) + lc * 8;
  }

  uint4 ra[A_IT], rb[B_IT];
  auto load_global = [&](int k0) {
    const bool kv = (k0 + lc * 8) < p.K;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) ra[i] = kv ? *(const uint4 *)(a_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < B_IT; ++i) rb[i] = kv ? *(const uint4 *)(w_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
  };
  auto store_lds = [&](int stage) {
    unsigned char *sa = smem + stage * STAGE_BYTES;
    unsigned char *sb = sa + BM * 128;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      int r = lr + i * ROWS_PER_IT;
      *(uint4 *)(sa + r * 128 + ((lc ^ ((r >> 1) & 7)) << 4)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      int r = lr + i * ROWS_PER_IT;
      *(uint4 *)(sb + r * 128 + ((lc ^ ((r >> 1) & 7)) << 4)) = rb[i];
    }
  };

  floatx16 acc[FN][FM];
#pragma unroll
  for (int bn = 0; bn < FN; ++bn)
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[bn][bm][v] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) load_global((kt + 1) * BK);
    const unsigned char *sa = smem + (kt & 1) * STAGE_BYTES;
    const unsigned char *sb = sa + BM * 128;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int cc = kk * 2 + g;
      bf16x8 wf[FN], af[FM];
#pragma unroll
      for (int bn = 0; bn < FN; ++bn) {
        int r = wn * WTN + bn * 32 + l32;
        wf[bn] = *(const bf16x8 *)(sb + r * 128 + ((cc ^ ((r >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int bm = 0; bm < FM; ++bm) {
        int r = wm * WTM + bm * 32 + l32;
        af[bm] = *(const bf16x8 *)(sa + r * 128 + ((cc ^ ((r >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int bn = 0; bn < FN; ++bn)
#pragma unroll
        for (int bm = 0; bm < FM; ++bm)
          acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[bn], af[bm], acc[bn][bm], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  gemm_epilogue<EPI, FM, FN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane);
}

// ---------------------------------------------------------------------------
// Epilogue that leaves through LDS.  The accumulator layout gives a lane 4
// consecutive columns of 32 different rows, i.e. 8-byte stores into 32 different
// cache lines per instruction.  Here each wave first applies its epilogue
// arithmetic in registers, writes the result into a private LDS slab laid out
// [row][column] (row stride padded by 16 bytes), and then streams it out with
// 16-byte stores in which 16 (or 8) consecutive lanes cover one contiguous row
// segment of 256 (128) bytes.  The residual add stages fp32 accumulators, 32 rows
// at a time, and adds them to the fp32 residual stream in place.
template <int EPI, int FM, int FN>
__device__ __forceinline__ void gemm_epilogue_lds(const GemmParams &p, floatx16 (&acc)[FN][FM], const int m_base,
                                                  const int n_base, const int lane, unsigned char *slab) {
  static_assert(FN == 4, "wave tile spans 128 output columns");
  const int l32 = lane & 31, g = lane >> 5;
  if (n_base >= p.N) return;                       // N is a multiple of 16; a wave tile past it has nothing to do
  if constexpr (EPI == EPI_RESID) {
    constexpr int RS = 128 * 4 + 16;               // fp32 row stride in bytes
    float *cbase = (float *)p.C + n_base;
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
#pragma unroll
      for (int bn = 0; bn < FN; ++bn)
#pragma unroll
        for (int jg = 0; jg < 4; ++jg)
          *(float4 *)(slab + l32 * RS + (bn * 32 + 8 * jg + 4 * g) * 4) =
              make_float4(acc[bn][bm][4 * jg], acc[bn][bm][4 * jg + 1], acc[bn][bm][4 * jg + 2], acc[bn][bm][4 * jg + 3]);
      // a wave's LDS operations execute in order: the reads below see the writes above
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row = it * 4 + (lane >> 4), ch = lane & 15;
        const int m = m_base + bm * 32 + row, n = n_base + ch * 8;
        const float4 lo = *(const float4 *)(slab + row * RS + ch * 32), hi = *(const float4 *)(slab + row * RS + ch * 32 + 16);
        if (m < p.M && n < p.N) {
          float4 *dst = (float4 *)(cbase + (int64_t)m * p.ldc + ch * 8);
          const float4 r0 = dst[0], r1 = dst[1];
          dst[0] = make_float4(r0.x + lo.x, r0.y + lo.y, r0.z + lo.z, r0.w + lo.w);
          dst[1] = make_float4(r1.x + hi.x, r1.y + hi.y, r1.z + hi.z, r1.w + hi.w);
        }
      }
    }
    return;
  } else {
    constexpr int NC = (EPI == EPI_SWIGLU) ? 64 : 128;   // output columns of the wave tile
    constexpr int RS = NC * 2 + 16;                      // bf16 row stride in bytes
    constexpr int CPR = NC / 8, RPI = 64 / CPR;          // 16-byte chunks per row, rows per store instruction
    // ---- epilogue arithmetic in registers, result (bf16) into the slab ----
    int kind = 0, col0 = n_base, proj = 0;               // QKV/KV: kind 0 = q, 1 = k, 2 = v
    if constexpr (EPI == EPI_QKV) {
      if (n_base < p.q_dim) { kind = 0; col0 = n_base; }
      else if (n_base < p.q_dim + p.kv_dim) { kind = 1; col0 = n_base - p.q_dim; }
      else { kind = 2; col0 = n_base - p.q_dim - p.kv_dim; }
    } else if constexpr (EPI == EPI_KV) {
      proj = n_base / (2 * p.kv_dim);
      const int within = n_base % (2 * p.kv_dim);
      kind = within < p.kv_dim ? 1 : 2;
      col0 = within % p.kv_dim;
    }
    const int hd = p.head_dim;
    float amax_h[2] = {0.f, 0.f};
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      const int m = m_base + bm * 32 + l32;
      const int mc = m < p.M ? m : p.M - 1;
      unsigned char *srow = slab + (bm * 32 + l32) * RS;
      if constexpr (EPI == EPI_SWIGLU) {
        const float rs = p.rstd ? p.rstd[mc] : 1.f;
#pragma unroll
        for (int bn = 0; bn < FN; ++bn)
#pragma unroll
          for (int jg = 0; jg < 2; ++jg) {
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float gt = acc[bn][bm][4 * jg + e] * rs, up = acc[bn][bm][4 * (jg + 2) + e] * rs;
              o[e] = gt * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * up;   // silu(gate) * up
            }
            *(uint2 *)(srow + (bn * 16 + 8 * jg + 4 * g) * 2) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
          }
      } else {
        if constexpr (EPI == EPI_QKV || EPI == EPI_KV) {
          const float rs = p.rstd ? p.rstd[mc] : 1.f;
#pragma unroll
          for (int bn = 0; bn < FN; ++bn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bn][bm][v] *= rs;
          if (kind != 2) {
            const float2 *cs = p.cos_sin + (int64_t)mc * (hd / 2);
            const int half_blocks = hd / 64, heads_per_tile = 128 / hd;
            for (int hh = 0; hh < heads_per_tile; ++hh)
              for (int hb = 0; hb < half_blocks; ++hb) {
                const int blo = hh * (hd / 32) + hb, bhi = blo + half_blocks;
#pragma unroll
                for (int jg = 0; jg < 4; ++jg) {
                  const int i0 = hb * 32 + 8 * jg + 4 * g;
                  const float4 c01 = *(const float4 *)(cs + i0), c23 = *(const float4 *)(cs + i0 + 2);
                  const float cv[4] = {c01.x, c01.z, c23.x, c23.z}, sv[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
                  for (int e = 0; e < 4; ++e) {
                    float x1 = 0.f, x2 = 0.f;
#pragma unroll
                    for (int b = 0; b < FN; ++b) {
                      if (b == blo) x1 = acc[b][bm][4 * jg + e];
                      if (b == bhi) x2 = acc[b][bm][4 * jg + e];
                    }
                    const float y1 = x1 * cv[e] - x2 * sv[e], y2 = x2 * cv[e] + x1 * sv[e];
#pragma unroll
                    for (int b = 0; b < FN; ++b) {
                      if (b == blo) acc[b][bm][4 * jg + e] = y1;
                      if (b == bhi) acc[b][bm][4 * jg + e] = y2;
                    }
                  }
                }
              }
          }
        }
#pragma unroll
        for (int bn = 0; bn < FN; ++bn)
#pragma unroll
          for (int jg = 0; jg < 4; ++jg) {
            const uint2 pk = make_uint2(pack_bf16x2(acc[bn][bm][4 * jg], acc[bn][bm][4 * jg + 1]), pack_bf16x2(acc[bn][bm][4 * jg + 2], acc[bn][bm][4 * jg + 3]));
            *(uint2 *)(srow + (bn * 32 + 8 * jg + 4 * g) * 2) = pk;
            if constexpr (EPI == EPI_QKV || EPI == EPI_KV) {
              if (p.amax && kind != 0 && m < p.M) {   // absmax of the values as stored (bf16-rounded)
                const float a = fmaxf(fmaxf(fabsf(bf16lo(pk.x)), fabsf(bf16hi(pk.x))), fmaxf(fabsf(bf16lo(pk.y)), fabsf(bf16hi(pk.y))));
                if ((bn * 32) / hd == 0) amax_h[0] = fmaxf(amax_h[0], a); else amax_h[1] = fmaxf(amax_h[1], a);
              }
            }
          }
      }
    }
    if constexpr (EPI == EPI_QKV || EPI == EPI_KV) {
      if (p.amax && kind != 0) {
        const int n_kv_heads = p.kv_dim / hd;
        for (int hh = 0; hh < 128 / hd; ++hh) {
          const float a = wave_max(amax_h[hh]);
          if (lane == 0)
            atomicMax(p.amax + ((int64_t)(p.first_cache_layer + proj) * 2 + (kind == 2 ? 1 : 0)) * n_kv_heads + col0 / hd + hh, __float_as_uint(a));
        }
      }
    }
    // ---- stream the slab out: lane -> (row it*RPI + lane/CPR, 16-byte chunk lane%CPR) ----
    // Destination selected once (uniform over the wave): base pointer and row stride in elements; the rows
    // of the paged cache go through p.slots, all read before the first store (loads and stores share one
    // counter: a load issued between stores would wait for the stores before it).
    const int ch = lane % CPR;
    bf16_t *obase;
    int64_t ostride;
    bool paged = false;
    if constexpr (EPI == EPI_STORE_BF16) { obase = (bf16_t *)p.C + n_base; ostride = p.ldc; }
    else if constexpr (EPI == EPI_SWIGLU) { obase = (bf16_t *)p.C + n_base / 2; ostride = p.ldc; }
    else if constexpr (EPI == EPI_QKV) {
      obase = p.q_out; ostride = p.q_dim;
      if (kind == 1) { obase = p.k_out; ostride = p.kv_dim; }
      if (kind == 2) { obase = p.v_out; ostride = p.kv_dim; }
      obase += col0;
    } else {
      obase = p.stage + n_base; ostride = p.N;
      if (!p.stage) {
        obase = p.cache + (int64_t)(p.first_cache_layer + proj) * p.cache_layer_stride + (kind == 2 ? p.cache_kv_stride : 0) + col0;
        ostride = p.kv_dim; paged = true;
      }
    }
    constexpr int N_IT = FM * 32 / RPI;
    int64_t orow[N_IT];
#pragma unroll
    for (int it = 0; it < N_IT; ++it) {
      const int m = m_base + it * RPI + lane / CPR;
      orow[it] = m;
      if constexpr (EPI == EPI_KV) { if (paged) orow[it] = p.slots[m < p.M ? m : p.M - 1]; }
    }
#pragma unroll
    for (int it = 0; it < N_IT; ++it) {
      const int row = it * RPI + lane / CPR;
      const int m = m_base + row;
      const uint4 val = *(const uint4 *)(slab + row * RS + ch * 16);
      if (m >= p.M) continue;
      if constexpr (EPI == EPI_STORE_BF16) { if (n_base + ch * 8 >= p.N) continue; }
      if constexpr (EPI == EPI_SWIGLU) { if (n_base + ch * 16 >= p.N) continue; }
      *(uint4 *)(obase + orow[it] * ostride + ch * 8) = val;
    }
  }
}

// ---------------------------------------------------------------------------
// Five-stage variant of the direct-to-LDS main loop with 32-wide k steps.
// LDS holds five (BM+BN) x 64-byte stages (160 KB for 256x256): while step t is
// multiplied, the loads of steps t+3 and t+4 are in flight and step t+1/t+2 are
// resident.  The LDS-DMA instructions of a step are spread one by one between
// its MFMAs (the address unit accepts about one 1 KB request per 16 cycles per
// CU, so a burst of them stalls the issuing waves), operand fragments of the
// next k sub-step are fetched between the MFMAs of the current one, including
// across the step boundary, and the only synchronisation is one barrier per
// step, which (a) publishes the step that landed two steps ahead and (b) frees
// the stage that the next step's loads overwrite.
// A stage row is 64 bytes = four 16-byte chunks; chunk c of row r sits at
// physical chunk c ^ ((r >> 2) & 3), which makes any 16 consecutive rows of one
// logical chunk hit 16 different bank groups.
// One LDS-DMA request: 64 lanes x 16 bytes from per-lane global addresses into the 1 KB of LDS
// starting at byte offset lds_addr (wave-uniform).  Written as inline assembly because the
// compiler, not knowing which LDS bytes a DMA targets, would otherwise wait for *all* outstanding
// loads before the next LDS read; here the waits are placed by hand (s_waitcnt vmcnt).
__device__ __forceinline__ void lds_dma16(const void *gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_dlds5_kernel(GemmParams p) {
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  static_assert(WTN == 128 && WTM % 32 == 0, "wave tile");
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int NS = 5, BKS = 32;                            // stages, k values per step
  constexpr int A_CH = BM / 16 / NW, B_CH = BN / 16 / NW;   // 1 KB chunks (16 rows) per wave per stage
  constexpr int LPW = A_CH + B_CH;                           // LDS-DMA loads per wave per step
  constexpr int STAGE_BYTES = (BM + BN) * 64;
  constexpr int NMF = FN * FM;                               // MFMAs per 16-wide sub-step
  constexpr int GSP = NMF / (LPW / 2);                       // MFMAs between two LDS-DMA requests of a wave
  static_assert(LPW % 2 == 0 && NMF % (LPW / 2) == 0 && FN + FM <= NMF, "interleave slots");

  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, g = lane >> 5;

  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= total) return;
  const int GM = p.raster_gm > 0 ? p.raster_gm : 8;
  const int group = logical / (GM * tiles_n);
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_group = logical % (GM * tiles_n);
  const int tm = first_m + in_group % gsz, tn = in_group / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  // LDS-DMA source: lane i of a 16-row chunk -> row i/4, logical chunk (i%4) ^ ((i/16)&3)
  const int cr = lane >> 2;
  const int cl = (lane & 3) ^ ((lane >> 4) & 3);
  const bf16_t *a_ptr[A_CH];
  const bf16_t *w_ptr[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    int m = m0 + (wave + i * NW) * 16 + cr;
    m = m < p.M ? m : p.M - 1;
    a_ptr[i] = p.A + (int64_t)m * p.lda + cl * 8;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    int n = n0 + (wave + i * NW) * 16 + cr;
    n = n < p.N ? n : p.N - 1;
    w_ptr[i] = (p.wtab ? p.wtab[n >> 4] + (int64_t)(n & 15) * p.ldw : p.W + (int64_t)n * p.ldw) + cl * 8;
  }
  typedef __attribute__((address_space(3))) void *lds_ptr_t;
  const unsigned lds_base = (unsigned)(size_t)(lds_ptr_t)smem;
  // one of the LPW loads of a step: idx < A_CH -> A chunk, else W chunk; `stage` = byte offset of the stage
  auto issue_one = [&](int idx, unsigned stage, int k0) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
      if (idx == i) lds_dma16(a_ptr[i] + k0, lds_base + stage + (wave + i * NW) * 1024);
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
      if (idx == A_CH + i) lds_dma16(w_ptr[i] + k0, lds_base + stage + BM * 64 + (wave + i * NW) * 1024);
  };

  floatx16 acc[FN][FM];
#pragma unroll
  for (int bn = 0; bn < FN; ++bn)
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[bn][bm][v] = 0.f;

  int w_off[FN], a_off[FM], w_sw[FN], a_sw[FM];
#pragma unroll
  for (int bn = 0; bn < FN; ++bn) { int r = wn * WTN + bn * 32 + l32; w_off[bn] = BM * 64 + r * 64; w_sw[bn] = (r >> 2) & 3; }
#pragma unroll
  for (int bm = 0; bm < FM; ++bm) { int r = wm * WTM + bm * 32 + l32; a_off[bm] = r * 64; a_sw[bm] = (r >> 2) & 3; }

  bf16x8 wf[2][FN], af[2][FM];
  // fragment idx (0..FN+FM-1) of sub-step kk from stage st into buffer buf
  auto load_frag = [&](int idx, int buf, const unsigned char *st, int kk) {
    const int cc = kk * 2 + g;
#pragma unroll
    for (int bn = 0; bn < FN; ++bn)
      if (idx == bn) wf[buf][bn] = *(const bf16x8 *)(st + w_off[bn] + ((cc ^ w_sw[bn]) << 4));
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
      if (idx == FN + bm) af[buf][bm] = *(const bf16x8 *)(st + a_off[bm] + ((cc ^ a_sw[bm]) << 4));
  };

  const int nk = p.K / BKS;
  // prologue: steps 0..3 in flight, steps 0 and 1 resident
#pragma unroll
  for (int s0 = 0; s0 < NS - 1; ++s0) {
    const int k0 = (s0 < nk ? s0 : nk - 1) * BKS;
#pragma unroll
    for (int i = 0; i < LPW; ++i) issue_one(i, s0 * STAGE_BYTES, k0);
  }
  constexpr int VMCNT = (NS - 3) * LPW;   // the NS-3 youngest groups may stay in flight
  __builtin_amdgcn_s_waitcnt(0x0F70 | (VMCNT & 15) | ((VMCNT >> 4) << 14));
  __syncthreads();
#pragma unroll
  for (int i = 0; i < FN + FM; ++i) load_frag(i, 0, smem, 0);

  int s_cur = 0;                 // stage of step t
  for (int t = 0; t < nk; ++t) {
    const int s_nxt = s_cur + 1 < NS ? s_cur + 1 : 0;           // stage of step t+1 (resident)
    const int s_ld = s_cur == 0 ? NS - 1 : s_cur - 1;           // stage of step t+4 = stage of step t-1 (free)
    const unsigned char *st = smem + s_cur * STAGE_BYTES;
    const unsigned char *stn = smem + s_nxt * STAGE_BYTES;
    const unsigned stl = s_ld * STAGE_BYTES;
    const int kl = (t + NS - 1 < nk ? t + NS - 1 : nk - 1) * BKS;   // clamped: the request count per step stays constant
    __builtin_amdgcn_sched_barrier(0);
    // sub-step 0: MFMAs on fragment buffer 0; fetch buffer 1 (sub-step 1 of this stage); first half of the loads
#pragma unroll
    for (int i = 0; i < NMF; ++i) {
      const int bn = i / FM, bm = i % FM;
      acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0][bn], af[0][bm], acc[bn][bm], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (i < FN + FM) load_frag(i, 1, st, 1);
      if ((i % GSP) == GSP - 1) issue_one(i / GSP, stl, kl);              // one request every GSP MFMAs: keeps the address unit's queue short
      __builtin_amdgcn_sched_barrier(0);
    }
    // sub-step 1: MFMAs on buffer 1; fetch buffer 0 from the next stage (resident since the previous barrier); second half of the loads
#pragma unroll
    for (int i = 0; i < NMF; ++i) {
      const int bn = i / FM, bm = i % FM;
      acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][bn], af[1][bm], acc[bn][bm], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (i < FN + FM) load_frag(i, 0, stn, 0);
      if ((i % GSP) == GSP - 1) issue_one(LPW / 2 + i / GSP, stl, kl);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70 | (VMCNT & 15) | ((VMCNT >> 4) << 14));   // step t+2 has landed (this wave's part)
    __syncthreads();
    s_cur = s_nxt;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the clamped extra loads ...
  __syncthreads();                      // ... of every wave, before LDS is reused by the epilogue
  constexpr int SLAB = WTM * (128 * 2 + 16) > 32 * (128 * 4 + 16) ? WTM * (128 * 2 + 16) : 32 * (128 * 4 + 16);
  static_assert(NW * SLAB <= 5 * STAGE_BYTES, "epilogue slabs must fit in the stage memory");
  unsigned char *slab = smem + wave * SLAB;
  if constexpr (EPI == EPI_STORE_F32) gemm_epilogue<EPI, FM, FN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane);
  else gemm_epilogue_lds<EPI, FM, FN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane, slab);
}

template <int BM, int BN, int WGM, int WGN, int EPI>
int launch_dlds5(const GemmParams &p, hipStream_t st) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int SMEM = 5 * (BM + BN) * 64;
  auto kern = gemm_dlds5_kernel<BM, BN, WGM, WGN, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  const int grid = ((tiles + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), SMEM, st, p);
  return 0;
}

template <int BM, int BN, int WGM, int WGN, int EPI>
int launch_one(const GemmParams &p, hipStream_t st) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int SMEM = 2 * (BM + BN) * 128;
  auto kern = gemm_kernel<BM, BN, WGM, WGN, EPI>;
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  const int grid = ((tiles + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), SMEM, st, p);
  return 0;
}

// ---------------------------------------------------------------------------
// Main loop that keeps the weight operand out of LDS.  The weights are static, so
// they can be stored once in MFMA fragment order (`wpack`: for every block of 32
// output rows and 16 k values, the 1 KB that the 64 lanes hold as first operand,
// lane i at byte 16*i).  A wave then fetches its weight fragments with fully
// coalesced 16-byte-per-lane loads straight into registers, four 64-wide k steps
// ahead, and LDS carries the activations only: five stages of 256 rows x 128
// bytes, filled by LDS-DMA in whole 128-byte row pieces, three steps ahead.
// The four waves sit side by side along N (wave tile 256 x 64), so no weight byte
// is loaded twice; every wave reads all of the activation tile from LDS (the same
// LDS read volume as a 2 x 2 arrangement of 128 x 128 wave tiles, half the LDS
// writes, half the LDS-DMA requests).  One barrier per 64-wide step, placed
// before the last 16-wide sub-step, where the next step's activations are first
// read.  Needs K % 256 == 0 (four register slots, statically indexed) and
// N % 256 == 0.
template <int EPI, int FM, bool NORM_OUT = false>   // NORM_OUT (RESID only): also the next projection's bf16 operand and the rows' sums of squares
__device__ __forceinline__ void gemm_epilogue_n64(const GemmParams &p, floatx16 (&acc)[2][FM], const int m_base,
                                                  const int n_base, const int lane, unsigned char *slab) {
  // acc[bn][bm][4*jg + e] is C[m_base + bm*32 + l32][n_base + bn*32 + 8*jg + 4*g + e].  32 rows at a
  // time go through a per-wave LDS slab (row stride padded by 16 bytes) and leave as 16-byte stores
  // in which consecutive lanes cover a contiguous row segment.
  const int l32 = lane & 31, g = lane >> 5;
  if constexpr (EPI == EPI_RESID) {
    // C (fp32, the residual stream) += acc.  Optionally also the bf16 operand of the next projection,
    // hb = bf16(C_new * gain of that projection's RMSNorm), and the sum of squares of C_new over this
    // wave's 64 columns (the consumer's epilogue applies 1/rms as a row factor).
    constexpr int RS = 64 * 4 + 16;                // fp32 row stride in bytes
    float *cbase = (float *)p.C + n_base;
    const int ch = lane & 7, r8 = lane >> 3;       // this lane's 8 columns, its row inside a group of 8
    float gv[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
    if (NORM_OUT && p.hb_gain) {
      const uint4 gq = *(const uint4 *)(p.hb_gain + n_base + ch * 8);
      gv[0] = bf16lo(gq.x); gv[1] = bf16hi(gq.x); gv[2] = bf16lo(gq.y); gv[3] = bf16hi(gq.y);
      gv[4] = bf16lo(gq.z); gv[5] = bf16hi(gq.z); gv[6] = bf16lo(gq.w); gv[7] = bf16hi(gq.w);
    }
    // The residual rows are requested for half of the wave tile at a time (128 registers; the operand
    // registers of the main loop are free by now), all of a half before its first store: loads and stores
    // share one counter, so a load issued between stores would wait for the stores before it.
    constexpr int HB = FM / 2;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      float4 res[HB][4][2];
#pragma unroll
      for (int b = 0; b < HB; ++b)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int m = m_base + (half * HB + b) * 32 + it * 8 + r8;
          const float4 *src = (const float4 *)(cbase + (int64_t)(m < p.M ? m : p.M - 1) * p.ldc + ch * 8);
          res[b][it][0] = src[0];
          res[b][it][1] = src[1];
        }
#pragma unroll
      for (int b = 0; b < HB; ++b) {
        const int bm = half * HB + b;
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
#pragma unroll
          for (int jg = 0; jg < 4; ++jg)
            *(float4 *)(slab + l32 * RS + (bn * 32 + 8 * jg + 4 * g) * 4) =
                make_float4(acc[bn][bm][4 * jg], acc[bn][bm][4 * jg + 1], acc[bn][bm][4 * jg + 2], acc[bn][bm][4 * jg + 3]);
        // a wave's LDS operations execute in order: the reads below see the writes above
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = it * 8 + r8;
          const int m = m_base + bm * 32 + row;
          const float4 lo = *(const float4 *)(slab + row * RS + ch * 32), hi = *(const float4 *)(slab + row * RS + ch * 32 + 16);
          const float4 r0 = res[b][it][0], r1 = res[b][it][1];
          const float x[8] = {r0.x + lo.x, r0.y + lo.y, r0.z + lo.z, r0.w + lo.w, r1.x + hi.x, r1.y + hi.y, r1.z + hi.z, r1.w + hi.w};
          if (m < p.M) {
            float4 *dst = (float4 *)(cbase + (int64_t)m * p.ldc + ch * 8);
            dst[0] = make_float4(x[0], x[1], x[2], x[3]);
            dst[1] = make_float4(x[4], x[5], x[6], x[7]);
            if constexpr (NORM_OUT)
              *(uint4 *)(p.hb + (int64_t)m * p.ldc + n_base + ch * 8) =
                  make_uint4(pack_bf16x2(x[0] * gv[0], x[1] * gv[1]), pack_bf16x2(x[2] * gv[2], x[3] * gv[3]),
                             pack_bf16x2(x[4] * gv[4], x[5] * gv[5]), pack_bf16x2(x[6] * gv[6], x[7] * gv[7]));
          }
          if constexpr (NORM_OUT) {   // fixed order: the lane's 8 columns left to right, then a butterfly over the row's 8 lanes
            float sq = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) sq += x[e] * x[e];
            sq += __shfl_xor(sq, 1);
            sq += __shfl_xor(sq, 2);
            sq += __shfl_xor(sq, 4);
            if (ch == 0 && m < p.M) p.ssq[(int64_t)m * (p.N >> 6) + (n_base >> 6)] = sq;
          }
        }
      }
    }
  } else if constexpr (EPI == EPI_QKV || EPI == EPI_KV) {
    // The wave's 64 (virtual) columns are one head (head_dim 64: blocks = first / second half) or, for
    // head_dim 128, half a head in the packed order: block 0 = columns s*32.. of the first half, block 1
    // = their rotary partners s*32 + 64.. (s = parity of the wave tile inside the head).  Either way
    // element v of block 0 and element v of block 1 are rotary partners.
    const int hd = p.head_dim;
    const int head_base = hd == 128 ? (n_base & ~127) : n_base;
    const int s = hd == 128 ? ((n_base >> 6) & 1) : 0;
    int kind, col0, proj = 0;                          // kind 0 = q, 1 = k, 2 = v; col0 = head's first column in its output
    if constexpr (EPI == EPI_QKV) {
      if (head_base < p.q_dim) { kind = 0; col0 = head_base; }
      else if (head_base < p.q_dim + p.kv_dim) { kind = 1; col0 = head_base - p.q_dim; }
      else { kind = 2; col0 = head_base - p.q_dim - p.kv_dim; }
    } else {
      proj = head_base / (2 * p.kv_dim);
      const int within = head_base % (2 * p.kv_dim);
      kind = within < p.kv_dim ? 1 : 2;
      col0 = within % p.kv_dim;
    }
    const int blk_stride = hd == 128 ? 64 : 32;        // real columns between block 0 and block 1
    constexpr int RS = 64 * 2 + 16;
    float amax_h = 0.f;
    // Destination of this wave's columns, selected once (uniform over the wave): base pointer of the
    // head's first column and the row stride in elements; rows of the paged cache go through p.slots.
    // (Selecting per store, through a table indexed by `kind`, cost a private-memory lookup, a full
    // vmcnt wait and a flat store for each of the 32 stores of a wave tile.)
    bf16_t *obase;
    int64_t ostride;
    bool paged = false;
    if constexpr (EPI == EPI_QKV) {
      obase = p.q_out; ostride = p.q_dim;
      if (kind == 1) { obase = p.k_out; ostride = p.kv_dim; }
      if (kind == 2) { obase = p.v_out; ostride = p.kv_dim; }
    } else {
      obase = p.stage + (int64_t)proj * 2 * p.kv_dim + (kind == 2 ? p.kv_dim : 0); ostride = p.N;
      if (!p.stage) {
        obase = p.cache + (int64_t)(p.first_cache_layer + proj) * p.cache_layer_stride + (kind == 2 ? p.cache_kv_stride : 0);
        ostride = p.kv_dim; paged = true;
      }
    }
    obase += col0 + s * 32;
    // 1/rms of this lane's rows, all requested before the first use (one latency, not one per 32 rows)
    float rsv[FM];
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      const int m = m_base + bm * 32 + l32;
      rsv[bm] = p.rstd ? p.rstd[m < p.M ? m : p.M - 1] : 1.f;
    }
    // Two passes, so that no load follows a store: loads and stores share one counter, and with both
    // kinds pending every wait for a load becomes a wait for everything, stores included (which made
    // each 32-row block of the epilogue wait for the previous block's stores to reach memory).
    // Pass 1: per 32-row block the cos/sin pieces (requested CSD - 1 blocks ahead: they are 32-row gathers
    // that mostly miss L2, and one block of arithmetic covers only a third of their latency) and, for the
    // paged cache, the rows' slots; rotation, rounding, bf16 rows into the wave's LDS slab (FM blocks of 32 rows).
    // Pass 2: the slab leaves as 16-byte stores in which consecutive lanes cover a contiguous row piece.
    constexpr int SLAB_BM = 32 * RS;   // bytes per 32-row block
    constexpr int CSD = (EPI == EPI_QKV) ? 4 : 2;   // the paged variant keeps 64 registers of slots instead
    float4 csb[CSD][8];
    auto load_cs = [&](int bm) {
      const int m = m_base + bm * 32 + l32;
      const float2 *cs = p.cos_sin + (int64_t)(m < p.M ? m : p.M - 1) * (hd / 2) + s * 32 + 4 * g;
#pragma unroll
      for (int jg = 0; jg < 4; ++jg) {
        csb[bm % CSD][2 * jg] = *(const float4 *)(cs + 8 * jg);
        csb[bm % CSD][2 * jg + 1] = *(const float4 *)(cs + 8 * jg + 2);
      }
    };
    if (kind != 2) {
#pragma unroll
      for (int b = 0; b < CSD - 1; ++b) load_cs(b);
    }
    int64_t orow[FM][4];   // output rows of this lane's stores (the paged cache: their slots)
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int mm = m_base + bm * 32 + it * 8 + (lane >> 3);
        orow[bm][it] = mm;
        if constexpr (EPI == EPI_KV) { if (paged) orow[bm][it] = p.slots[mm < p.M ? mm : p.M - 1]; }
      }
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      const int m = m_base + bm * 32 + l32;
      const float rs = rsv[bm];
      unsigned char *srow = slab + bm * SLAB_BM + l32 * RS;
      if (kind != 2 && bm + CSD - 1 < FM) load_cs(bm + CSD - 1);
#pragma unroll
      for (int jg = 0; jg < 4; ++jg) {
        float y1[4], y2[4];
        const int i0 = 8 * jg + 4 * g;
        float cv[4] = {1.f, 1.f, 1.f, 1.f}, sv[4] = {0.f, 0.f, 0.f, 0.f};
        if (kind != 2) {
          const float4 c01 = csb[bm % CSD][2 * jg], c23 = csb[bm % CSD][2 * jg + 1];
          cv[0] = c01.x; cv[1] = c01.z; cv[2] = c23.x; cv[3] = c23.z;
          sv[0] = c01.y; sv[1] = c01.w; sv[2] = c23.y; sv[3] = c23.w;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x1 = acc[0][bm][4 * jg + e] * rs, x2 = acc[1][bm][4 * jg + e] * rs;
          y1[e] = x1 * cv[e] - x2 * sv[e];
          y2[e] = x2 * cv[e] + x1 * sv[e];
        }
        const uint2 p1 = make_uint2(pack_bf16x2(y1[0], y1[1]), pack_bf16x2(y1[2], y1[3]));
        const uint2 p2 = make_uint2(pack_bf16x2(y2[0], y2[1]), pack_bf16x2(y2[2], y2[3]));
        *(uint2 *)(srow + i0 * 2) = p1;
        *(uint2 *)(srow + (32 + i0) * 2) = p2;
        if (p.amax && kind != 0 && m < p.M) {   // absmax of the values as stored (bf16-rounded)
          const float a1 = fmaxf(fmaxf(fabsf(bf16lo(p1.x)), fabsf(bf16hi(p1.x))), fmaxf(fabsf(bf16lo(p1.y)), fabsf(bf16hi(p1.y))));
          const float a2 = fmaxf(fmaxf(fabsf(bf16lo(p2.x)), fabsf(bf16hi(p2.x))), fmaxf(fabsf(bf16lo(p2.y)), fabsf(bf16hi(p2.y))));
          amax_h = fmaxf(amax_h, fmaxf(a1, a2));
        }
      }
    }
    // a wave's LDS operations execute in order: the reads below see the writes above
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
#pragma unroll
      for (int it = 0; it < 4; ++it) {   // 8 rows per instruction, chunk ch = 8 local columns; local block ch/4
        const int row = it * 8 + (lane >> 3), ch = lane & 7;
        const int mm = m_base + bm * 32 + row;
        const uint4 val = *(const uint4 *)(slab + bm * SLAB_BM + row * RS + ch * 16);
        if (mm < p.M) *(uint4 *)(obase + orow[bm][it] * ostride + (ch >> 2) * blk_stride + (ch & 3) * 8) = val;
      }
    if (p.amax && kind != 0) {
      const float a = wave_max(amax_h);
      if (lane == 0)
        atomicMax(p.amax + ((int64_t)(p.first_cache_layer + proj) * 2 + (kind == 2 ? 1 : 0)) * (p.kv_dim / hd) + col0 / hd, __float_as_uint(a));
    }
  } else {
    static_assert(EPI == EPI_STORE_BF16 || EPI == EPI_SWIGLU, "epilogues of the 64-column wave tile");
    constexpr int NC = (EPI == EPI_SWIGLU) ? 32 : 64;   // output columns of the wave tile
    constexpr int RS = NC * 2 + 16;                      // bf16 row stride in bytes
    constexpr int CPR = NC / 8, RPI = 64 / CPR;          // 16-byte chunks per row, rows per store instruction
    float rsv[FM];
    if constexpr (EPI == EPI_SWIGLU) {   // 1/rms of this lane's rows, all requested before the first use
#pragma unroll
      for (int bm = 0; bm < FM; ++bm) {
        const int m = m_base + bm * 32 + l32;
        rsv[bm] = p.rstd ? p.rstd[m < p.M ? m : p.M - 1] : 1.f;
      }
    }
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) {
      unsigned char *srow = slab + l32 * RS;
      if constexpr (EPI == EPI_SWIGLU) {
        const float rs = rsv[bm];
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
#pragma unroll
          for (int jg = 0; jg < 2; ++jg) {
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float gt = acc[bn][bm][4 * jg + e] * rs, up = acc[bn][bm][4 * (jg + 2) + e] * rs;
              o[e] = gt * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * up;   // silu(gate) * up
            }
            *(uint2 *)(srow + (bn * 16 + 8 * jg + 4 * g) * 2) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
          }
      } else {
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
#pragma unroll
          for (int jg = 0; jg < 4; ++jg)
            *(uint2 *)(srow + (bn * 32 + 8 * jg + 4 * g) * 2) =
                make_uint2(pack_bf16x2(acc[bn][bm][4 * jg], acc[bn][bm][4 * jg + 1]), pack_bf16x2(acc[bn][bm][4 * jg + 2], acc[bn][bm][4 * jg + 3]));
      }
      const int ch = lane % CPR;
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int row = it * RPI + lane / CPR;
        const int m = m_base + bm * 32 + row;
        const uint4 val = *(const uint4 *)(slab + row * RS + ch * 16);
        if (m >= p.M) continue;
        bf16_t *dst = (bf16_t *)p.C + (int64_t)m * p.ldc + (EPI == EPI_SWIGLU ? n_base / 2 : n_base);
        *(uint4 *)(dst + ch * 8) = val;
      }
    }
  }
}

template <int EPI, bool NORM_OUT = false>
__global__ __launch_bounds__(256) void gemm_wreg_kernel(GemmParams p) {
  constexpr int BM = 256, BN = 256, FM = 8;
  constexpr int NSA = 5, STAGE = BM * 128;   // activation stages: 256 rows x 128 bytes (one 64-wide k step)
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;

  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = p.N / BN;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= total) return;
  const int GM = p.raster_gm > 0 ? p.raster_gm : 8;
  const int group = logical / (GM * tiles_n);
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_group = logical % (GM * tiles_n);
  const int tm = first_m + in_group % gsz, tn = in_group / gsz;
  const int m0 = tm * BM, n0 = tn * BN + wave * 64;   // n0: first column of this wave

  // LDS-DMA sources: request i of this wave covers rows (wave*8 + i)*8 .. +7 of the tile, 128 bytes each;
  // this lane fetches row +(lane>>3), the 16-byte chunk that lands at physical chunk lane&7
  const bf16_t *a_ptr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (wave * 8 + i) * 8 + (lane >> 3);
    int m = m0 + r;
    m = m < p.M ? m : p.M - 1;
    a_ptr[i] = p.A + (int64_t)m * p.lda + (((lane & 7) ^ ((r >> 1) & 7)) * 8);
  }
  // packed weight fragments of the wave's two 32-row blocks: (block, k16) at ((block * K/16) + k16) * 512 elements
  const bf16_t *w_ptr[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) w_ptr[nb] = p.wpack + ((int64_t)(n0 / 32 + nb) * (p.K / 16)) * 512 + lane * 8;

  typedef __attribute__((address_space(3))) void *lds_ptr_t;
  const unsigned lds_base = (unsigned)(size_t)(lds_ptr_t)smem;

  floatx16 acc[2][FM];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[nb][bm][v] = 0.f;

  // activation fragment of m block bm, sub-step kk: row bm*32 + l32, chunk (2*kk + g) ^ swizzle(row);
  // the swizzle of a 128-byte row is (row >> 1) & 7, the same for every m block, and kk enters as an XOR with 32*kk
  const unsigned a_lane = l32 * 128 + ((g ^ ((l32 >> 1) & 7)) << 4);

  bf16x8 wf[4][8];   // [slot of the step][2*kk + nb]
  bf16x8 af[2][FM];
  const int nk = p.K / 64;

  auto issue_a = [&](int i, int stage, int step) {
    lds_dma16(a_ptr[i] + (int64_t)step * 64, lds_base + stage * STAGE + (wave * 8 + i) * 1024);
  };
  // Plain loads: the compiler places their vmcnt waits.  It counts only these loads, not the LDS-DMA
  // requests issued from inline assembly in between, so its waits are stricter than necessary, never
  // weaker.  (Hand-placed waits that relied on register loads and LDS-DMA completing in one common
  // order gave results that changed from run to run: the two kinds do not complete in issue order
  // relative to each other.)
  auto load_w = [&](bf16x8 &dst, int nb, int kk, int step) {
    dst = *(const bf16x8 *)(w_ptr[nb] + ((int64_t)step * 4 + kk) * 512);
  };

  // prologue: steps 0, 1, 2 requested (16 requests per wave and step, activations and weights alternating)
#pragma unroll
  for (int s0 = 0; s0 < 3; ++s0) {
    const int step = s0 < nk ? s0 : nk - 1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      issue_a(i, s0, step);
      load_w(wf[s0][i], i & 1, i >> 1, step);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16): step 0 has landed (this wave's part; at most the 16 LDS-DMA requests of steps 1, 2 remain)
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int bm = 0; bm < FM; ++bm) af[0][bm] = *(const bf16x8 *)(smem + a_lane + bm * 4096);

  int sa = 0;   // stage of the current step
  auto step_fn = [&](auto slot_c, const int it) {
    constexpr int slot = decltype(slot_c)::value;
    constexpr int lslot = (slot + 3) & 3;                 // the slot freed by the previous step takes the weights of step it+3
    const int sn = sa == NSA - 1 ? 0 : sa + 1;            // stage of step it+1
    const int sld = sa >= 2 ? sa - 2 : sa + 3;            // stage of step it+3 = stage of step it-2 (free)
    const int kl = it + 3 < nk ? it + 3 : nk - 1;         // clamped: the request count per step stays constant
    const unsigned char *st = smem + sa * STAGE, *stn = smem + sn * STAGE;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk == 3) {
        // Step it+1 (requested during step it-2) must be resident before its first fragments are read.
        // 14 LDS-DMA requests are younger than it (8 of step it-1, 6 of this step).  Register loads and
        // LDS-DMA do not complete in one common order, so all 14 requests that may stay in flight could
        // be LDS-DMA ones: the wait is for 14 in total, not for 14 + the 14 younger weight loads.
        __builtin_amdgcn_s_waitcnt(0x0F7E);   // vmcnt(14)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int nb = i / 8, bm = i % 8;
        acc[nb][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][kk * 2 + nb], af[kk & 1][bm], acc[nb][bm], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (i < 8) af[(kk + 1) & 1][i] = *(const bf16x8 *)((kk < 3 ? st : stn) + (a_lane ^ (unsigned)(((kk + 1) & 3) * 32)) + i * 4096);
        if (i % 8 == 3) issue_a(kk * 2 + i / 8, sld, kl);
        if (i % 8 == 7) load_w(wf[lslot][kk * 2 + i / 8], i / 8, kk, kl);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    sa = sn;
  };
  for (int it = 0; it < nk; it += 4) {
    step_fn(std::integral_constant<int, 0>{}, it);
    step_fn(std::integral_constant<int, 1>{}, it + 1);
    step_fn(std::integral_constant<int, 2>{}, it + 2);
    step_fn(std::integral_constant<int, 3>{}, it + 3);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the clamped extra requests ...
  __builtin_amdgcn_s_barrier();         // ... of every wave, before LDS is reused by the epilogue
  // per-wave slab: one 32-row block of fp32 (272-byte rows), or, for the rotating epilogues, all eight blocks of bf16 (144-byte rows)
  unsigned char *slab = smem + wave * ((EPI == EPI_QKV || EPI == EPI_KV) ? FM * 32 * (64 * 2 + 16) : 32 * (64 * 4 + 16));
  gemm_epilogue_n64<EPI, FM, NORM_OUT>(p, acc, m0, n0, lane, slab);
}

template <int EPI, bool NORM_OUT>
int launch_wreg_k(const GemmParams &p, hipStream_t st) {
  constexpr int SMEM = 5 * 256 * 128;
  auto kern = gemm_wreg_kernel<EPI, NORM_OUT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  const int tiles = ((p.M + 255) / 256) * (p.N / 256);
  hipLaunchKernelGGL(kern, dim3(((tiles + 7) / 8) * 8), dim3(256), SMEM, st, p);
  return 0;
}
template <int EPI>
int launch_wreg(const GemmParams &p, hipStream_t st) {
  if constexpr (EPI == EPI_RESID) {
    if (p.hb && p.ssq) return launch_wreg_k<EPI, true>(p, st);
  }
  return launch_wreg_k<EPI, false>(p, st);
}

// variant: 0 = pick by shape; 1 = 256x256 tile, register-staged loads; 2 = 128x128 tile; 14 / 15 = the
// five-stage direct-to-LDS loop with 4 / 8 waves; 27 = the packed-weight loop (needs p.wpack)
template <int EPI>
int launch_epi(const GemmParams &p, int variant, hipStream_t st) {
  if (variant == 0) variant = (p.M >= 1024) ? ((p.K % BK) == 0 ? 14 : 1) : 2;
  if constexpr (EPI != EPI_STORE_F32) {
    // weights available in fragment order: the loop that keeps them out of LDS
    if ((variant == 27 || variant == 14) && gemm_uses_packed_weights(p)) return launch_wreg<EPI>(p, st);
  }
  if (variant == 27) variant = 14;
  if ((variant == 14 || variant == 15) && (p.K % BK) != 0) variant = 1;
  if (variant == 14) return launch_dlds5<256, 256, 2, 2, EPI>(p, st);
  if (variant == 15) return launch_dlds5<256, 256, 4, 2, EPI>(p, st);
  if (variant == 1) return launch_one<256, 256, 2, 2, EPI>(p, st);
  return launch_one<128, 128, 4, 1, EPI>(p, st);
}

}  // namespace

// ---------------------------------------------------------------------------
// The rate the matrix unit sustains on given data (the chip is power-limited: it depends on the
// operand bits): every wave keeps 4 + 4 operand fragments of the caller's data in registers and
// issues 16 independent MFMAs per iteration into 16 accumulator tiles.
__global__ __launch_bounds__(256) void mfma_rate_kernel(const bf16_t *operands, float *sink, int iters) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {   // 8 KB per wave, 32 KB per workgroup, the same for every workgroup
    a[i] = *(const bf16x8 *)(operands + ((wave * 8 + i) * 64 + lane) * 8);
    b[i] = *(const bf16x8 *)(operands + ((wave * 8 + 4 + i) * 64 + lane) * 8);
  }
  floatx16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}
int launch_mfma_rate(const bf16_t *operands, float *sink, int32_t n_workgroups, int32_t iters, hipStream_t st) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(n_workgroups), dim3(256), 0, st, operands, sink, iters);
  return 0;
}

// Whether launch_gemm(p, epi, 0, ...) reads the fragment-order copy p.wpack (and not p.W / p.wtab): the
// driver needs to know, because that copy of a projection behind an RMSNorm has the norm's gain folded in.
bool gemm_uses_packed_weights(const GemmParams &p) {
  return p.wpack && p.M >= 1024 && (p.K % 256) == 0 && (p.N % 256) == 0;
}

int launch_gemm(const GemmParams &p, int epi, int variant, hipStream_t st) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return 0;
  switch (epi) {
    case EPI_STORE_BF16: return launch_epi<EPI_STORE_BF16>(p, variant, st);
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(p, variant, st);
    case EPI_RESID: return launch_epi<EPI_RESID>(p, variant, st);
    case EPI_SWIGLU: return launch_epi<EPI_SWIGLU>(p, variant, st);
    case EPI_QKV: return launch_epi<EPI_QKV>(p, variant, st);
    case EPI_KV: return launch_epi<EPI_KV>(p, variant, st);
  }
  return -1;
}
