// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T  with fused prologue
// (per-column RMSNorm gain on A) and epilogues (residual add, SwiGLU, rstd row
// scale + RoPE + q/k/v split, rstd + RoPE + paged KV scatter).
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
          } else {
            bf16_t *dst = (bf16_t *)p.C + (int64_t)m * p.ldc + n;
            if constexpr (EPI == EPI_RESID) {
              uint2 r = *(const uint2 *)dst;
              x0 += bf16lo(r.x); x1 += bf16hi(r.x); x2 += bf16lo(r.y); x3 += bf16hi(r.y);
            }
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
            o[e] = gt / (1.f + __expf(-gt)) * up;
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
      bf16_t *dst;
      if constexpr (EPI == EPI_QKV) {
        dst = kind == 0 ? p.q_out + (int64_t)mc * p.q_dim + col0
                        : (kind == 1 ? p.k_out : p.v_out) + (int64_t)mc * p.kv_dim + col0;
      } else {
        if (p.stage) dst = p.stage + (int64_t)mc * p.N + n_base;
        else dst = p.cache + (int64_t)(p.first_cache_layer + proj) * p.cache_layer_stride +
                   (kind == 2 ? p.cache_kv_stride : 0) + p.slots[mc] * p.kv_dim + col0;
      }
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

template <int BM, int BN, int WGM, int WGN, int EPI, bool GAIN>
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
  const bf16_t *g_ptr = nullptr;
  if constexpr (GAIN) g_ptr = p.gain_tab[n0 / p.gain_seg] + lc * 8;

  uint4 ra[A_IT], rb[B_IT];
  auto load_global = [&](int k0) {
    const bool kv = (k0 + lc * 8) < p.K;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) ra[i] = kv ? *(const uint4 *)(a_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < B_IT; ++i) rb[i] = kv ? *(const uint4 *)(w_ptr[i] + k0) : make_uint4(0, 0, 0, 0);
    if constexpr (GAIN) {
      uint4 gv = kv ? *(const uint4 *)(g_ptr + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        ra[i].x = pack_bf16x2(bf16lo(ra[i].x) * bf16lo(gv.x), bf16hi(ra[i].x) * bf16hi(gv.x));
        ra[i].y = pack_bf16x2(bf16lo(ra[i].y) * bf16lo(gv.y), bf16hi(ra[i].y) * bf16hi(gv.y));
        ra[i].z = pack_bf16x2(bf16lo(ra[i].z) * bf16lo(gv.z), bf16hi(ra[i].z) * bf16hi(gv.z));
        ra[i].w = pack_bf16x2(bf16lo(ra[i].w) * bf16lo(gv.w), bf16hi(ra[i].w) * bf16hi(gv.w));
      }
    }
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
// Main loop with direct global -> LDS loads (global_load_lds_dwordx4).  One
// instruction moves 64 x 16 bytes into 1 KB of LDS = 8 tile rows; lane i lands
// in (row i/8, physical chunk i%8), so it fetches the logical chunk
// (i%8) ^ ((row >> 1) & 7) of that row, which reproduces the XOR swizzle the
// MFMA operand reads expect.
// No staging registers and no LDS store instructions; needs K % 64 == 0 and no
// gain prologue.
template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_dlds_kernel(GemmParams p) {
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  static_assert(WTN == 128 && WTM % 32 == 0, "wave tile");
  constexpr int FM = WTM / 32, FN = WTN / 32;
  constexpr int A_CH = BM / 8 / NW, B_CH = BN / 8 / NW;   // 1 KB chunks per wave per stage
  constexpr int STAGE_BYTES = (BM + BN) * 128;

  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, g = lane >> 5;

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

  // lane -> (row within an 8-row chunk, logical 16-byte chunk)
  static_assert(NW % 2 == 0, "chunk parity must be a per-wave constant");
  const int cr = lane >> 3;                                   // row inside the wave's 8-row chunk
  const int cl = (lane & 7) ^ (((wave & 1) << 2) | (cr >> 1));  // ((8*chunk + cr) >> 1) & 7, chunk = wave + i*NW
  const bf16_t *a_ptr[A_CH];
  const bf16_t *w_ptr[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    int m = m0 + (wave + i * NW) * 8 + cr;
    m = m < p.M ? m : p.M - 1;
    a_ptr[i] = p.A + (int64_t)m * p.lda + cl * 8;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    int n = n0 + (wave + i * NW) * 8 + cr;
    n = n < p.N ? n : p.N - 1;
    w_ptr[i] = (p.wtab ? p.wtab[n >> 4] + (int64_t)(n & 15) * p.ldw : p.W + (int64_t)n * p.ldw) + cl * 8;
  }
  typedef __attribute__((address_space(3))) void *lds_ptr_t;
  typedef const __attribute__((address_space(1))) void *glb_ptr_t;
  auto issue_loads = [&](int stage, int k0) {
    unsigned char *sa = smem + stage * STAGE_BYTES;
    unsigned char *sb = sa + BM * 128;
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(a_ptr[i] + k0), (lds_ptr_t)(sa + (wave + i * NW) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(w_ptr[i] + k0), (lds_ptr_t)(sb + (wave + i * NW) * 1024), 16, 0, 0);
  };

  // L2 prefetch two k-tiles ahead: a 4-byte LDS-DMA read of the first word of
  // every 128-byte row segment of that tile, dumped into a scratch corner of LDS.
  // It costs no registers, pulls the lines into L2 early, and - because vector
  // loads retire in order - the end-of-tile wait can leave exactly these
  // youngest requests outstanding (vmcnt(PF)).
  constexpr int PF = (BM + BN) / (NW * 64);   // prefetch instructions per wave per tile
  const bf16_t *pf_ptr[PF];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    const int row = tid + i * NW * 64;        // 0..BM-1: A rows, BM..BM+BN-1: W rows
    if (row < BM) {
      int m = m0 + row;
      m = m < p.M ? m : p.M - 1;
      pf_ptr[i] = p.A + (int64_t)m * p.lda;
    } else {
      int n = n0 + row - BM;
      n = n < p.N ? n : p.N - 1;
      pf_ptr[i] = p.wtab ? p.wtab[n >> 4] + (int64_t)(n & 15) * p.ldw : p.W + (int64_t)n * p.ldw;
    }
  }
  unsigned char *pf_lds = smem + 2 * STAGE_BYTES + wave * 256;
  auto prefetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < PF; ++i) __builtin_amdgcn_global_load_lds((glb_ptr_t)(pf_ptr[i] + k0), (lds_ptr_t)pf_lds, 4, 0, 0);
  };

  floatx16 acc[FN][FM];
#pragma unroll
  for (int bn = 0; bn < FN; ++bn)
#pragma unroll
    for (int bm = 0; bm < FM; ++bm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[bn][bm][v] = 0.f;

  // byte offsets of this lane's operand rows inside a stage (row r, chunk c at r*128 + ((c ^ ((r>>1)&7)) << 4))
  int w_off[FN], a_off[FM], w_sw[FN], a_sw[FM];
#pragma unroll
  for (int bn = 0; bn < FN; ++bn) { int r = wn * WTN + bn * 32 + l32; w_off[bn] = BM * 128 + r * 128; w_sw[bn] = (r >> 1) & 7; }
#pragma unroll
  for (int bm = 0; bm < FM; ++bm) { int r = wm * WTM + bm * 32 + l32; a_off[bm] = r * 128; a_sw[bm] = (r >> 1) & 7; }

  bf16x8 wf[2][FN], af[2][FM];
  auto load_frags = [&](int buf, const unsigned char *st, int kk) {
    const int cc = kk * 2 + g;
#pragma unroll
    for (int bn = 0; bn < FN; ++bn) wf[buf][bn] = *(const bf16x8 *)(st + w_off[bn] + ((cc ^ w_sw[bn]) << 4));
#pragma unroll
    for (int bm = 0; bm < FM; ++bm) af[buf][bm] = *(const bf16x8 *)(st + a_off[bm] + ((cc ^ a_sw[bm]) << 4));
  };

  const int nk = p.K / BK;
  const bool use_pf = p.dbg != 4;
  issue_loads(0, 0);
  if (nk > 1 && use_pf) prefetch(BK);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk && p.dbg != 1) issue_loads((kt + 1) & 1, p.dbg == 2 ? 0 : (kt + 1) * BK);
    // always issued (clamped to the last tile) so that the vmcnt below is a constant
    if (use_pf) prefetch((kt + 2 < nk ? kt + 2 : nk - 1) * BK);
    const unsigned char *st = smem + (kt & 1) * STAGE_BYTES;
    load_frags(0, st, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      // Operands of step kk+1 are requested right after the first MFMAs of step
      // kk were issued, so at the top of every step the only outstanding LDS
      // reads are the ones it needs, and they have had most of a step to arrive.
#pragma unroll
      for (int bm = 0; bm < FM; ++bm)
        acc[0][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk & 1][0], af[kk & 1][bm], acc[0][bm], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (kk + 1 < BK / 16) load_frags((kk + 1) & 1, st, kk + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int bn = 1; bn < FN; ++bn)
#pragma unroll
        for (int bm = 0; bm < FM; ++bm)
          acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk & 1][bn], af[kk & 1][bm], acc[bn][bm], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // this wave's loads of the next tile have landed in LDS; the PF prefetches issued after them may still fly
    if (use_pf) __builtin_amdgcn_s_waitcnt(0x0F70 | PF); else __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the last prefetches before LDS is released
  gemm_epilogue<EPI, FM, FN>(p, acc, m0 + wm * WTM, n0 + wn * WTN, lane);
}

template <int BM, int BN, int WGM, int WGN, int EPI>
int launch_dlds(const GemmParams &p, hipStream_t st) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int SMEM = 2 * (BM + BN) * 128 + WGM * WGN * 256;   // two stages + prefetch scratch
  auto kern = gemm_dlds_kernel<BM, BN, WGM, WGN, EPI>;
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

template <int BM, int BN, int WGM, int WGN, int EPI, bool GAIN>
int launch_one(const GemmParams &p, hipStream_t st) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int SMEM = 2 * (BM + BN) * 128;
  auto kern = gemm_kernel<BM, BN, WGM, WGN, EPI, GAIN>;
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

template <int EPI, bool GAIN>
int launch_epi(const GemmParams &p, int variant, hipStream_t st) {
  if (variant == 0) variant = (p.M >= 1024) ? ((!GAIN && (p.K % BK) == 0) ? 5 : 1) : 2;
  if constexpr (!GAIN) {
    if ((variant == 4 || variant == 5) && (p.K % BK) != 0) variant = 1;
    if (variant == 4) return launch_dlds<256, 256, 4, 2, EPI>(p, st);
    if (variant == 5) return launch_dlds<256, 256, 2, 2, EPI>(p, st);
  }
  if (variant == 1 || variant == 4 || variant == 5) return launch_one<256, 256, 2, 2, EPI, GAIN>(p, st);
  return launch_one<128, 128, 4, 1, EPI, GAIN>(p, st);
}

}  // namespace

int launch_gemm(const GemmParams &p, int epi, int variant, hipStream_t st) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return 0;
  const bool gain = p.gain_tab != nullptr;
  switch (epi) {
    case EPI_STORE_BF16: return launch_epi<EPI_STORE_BF16, false>(p, variant, st);
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32, false>(p, variant, st);
    case EPI_RESID: return launch_epi<EPI_RESID, false>(p, variant, st);
    case EPI_SWIGLU: return gain ? launch_epi<EPI_SWIGLU, true>(p, variant, st) : launch_epi<EPI_SWIGLU, false>(p, variant, st);
    case EPI_QKV: return gain ? launch_epi<EPI_QKV, true>(p, variant, st) : launch_epi<EPI_QKV, false>(p, variant, st);
    case EPI_KV: return gain ? launch_epi<EPI_KV, true>(p, variant, st) : launch_epi<EPI_KV, false>(p, variant, st);
  }
  return -1;
}
