// Attention kernels for gfx950.
//
// 1. attn_prefill_kernel: causal grouped-query flash attention over packed fresh
//    sequences.  A workgroup (4 waves) owns 128 consecutive queries of one
//    (sequence, query head); each wave owns 32 queries.  K tiles [64 keys][hd]
//    and V^T tiles [hd][64 keys] are staged through LDS (double buffered).
//    Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16,
//    so one lane owns one query column: the running max / sum of the online
//    softmax are per-lane scalars (one cross-half exchange), and the exponentials
//    are already laid out as the second operand of O^T += V^T P^T.
// 2. attn_decode_kernel: one query row against a paged (bf16 or FP8) cache,
//    split over key ranges; used for the last-token tail and for decode tokens.
#include "common.h"

namespace {

constexpr int BQ = 128;   // queries per workgroup
constexpr int BKV = 64;   // keys per tile

template <int HD, bool PROF = false>
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(AttnPrefillParams p) {
  constexpr int KROW = HD * 2 + 16;        // padded K row bytes (conflict-free 16-byte reads)
  constexpr int VROW = BKV * 2 + 8;        // padded V^T row bytes (conflict-free 8-byte reads)
  constexpr int K_BYTES = BKV * KROW, V_BYTES = HD * VROW;
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int DS = HD / 16;              // d steps of the QK^T contraction
  constexpr int DB = HD / 32;              // 32-wide d blocks of the output
  constexpr int KCH = HD / 8;              // 16-byte chunks per K row
  constexpr int K_IT = BKV * KCH / 256;    // K chunks per thread
  constexpr int V_IT = HD * 8 / 256;       // V^T chunks per thread (rows of 8 chunks)

  extern __shared__ __align__(16) unsigned char smem[];

  const QBlock qb = p.qblocks[blockIdx.x];
  const int head = blockIdx.y;
  const int kvh = head / (p.n_q_heads / p.n_kv_heads);
  const int q_dim = p.n_q_heads * HD, kv_dim = p.n_kv_heads * HD;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;

  // ---- this lane's query: position and Q fragments (second MFMA operand) ----
  const int qpos = qb.q0 + wave * 32 + l32;            // position in the sequence
  const bool qvalid = qpos < qb.n;
  const int qrow = qb.row0 + wave * 32 + l32;
  const int qrow_c = qvalid ? qrow : qb.seq_row0 + qb.n - 1;
  bf16x8 qf[DS];
  {
    const bf16_t *qp = p.q + (int64_t)qrow_c * q_dim + head * HD;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) qf[ds] = *(const bf16x8 *)(qp + (ds * 2 + g) * 8);
  }

  // keys needed by the workgroup: 0 .. min(n, q0 + BQ) - 1
  const int k_end = (qb.q0 + BQ) < qb.n ? (qb.q0 + BQ) : qb.n;
  const int n_tiles = (k_end + BKV - 1) / BKV;
  const int wave_last = qb.q0 + wave * 32 + 31;       // last query position of this wave

  const bf16_t *kbase = p.k + (int64_t)qb.seq_row0 * kv_dim + kvh * HD;
  const bf16_t *vbase = p.vt + (int64_t)(kvh * HD) * p.vt_ld + qb.vt_col0;

  uint4 rk[K_IT], rv[V_IT];
  auto load_tile = [&](int t) {
    const int key0 = t * BKV;
#pragma unroll
    for (int i = 0; i < K_IT; ++i) {
      int idx = tid + i * 256;
      int r = idx / KCH, c = idx % KCH;
      int key = key0 + r;
      key = key < qb.n ? key : qb.n - 1;   // rows past the end are masked later; any finite data will do
      rk[i] = *(const uint4 *)(kbase + (int64_t)key * kv_dim + c * 8);
    }
#pragma unroll
    for (int i = 0; i < V_IT; ++i) {
      int idx = tid + i * 256;
      int d = idx / 8, c = idx % 8;
      rv[i] = *(const uint4 *)(vbase + (int64_t)d * p.vt_ld + key0 + c * 8);   // padded columns are zero
    }
  };
  auto store_tile = [&](int stage) {
    unsigned char *sk = smem + stage * STAGE;
    unsigned char *sv = sk + K_BYTES;
#pragma unroll
    for (int i = 0; i < K_IT; ++i) {
      int idx = tid + i * 256;
      int r = idx / KCH, c = idx % KCH;
      *(uint4 *)(sk + r * KROW + c * 16) = rk[i];
    }
#pragma unroll
    for (int i = 0; i < V_IT; ++i) {
      int idx = tid + i * 256;
      int d = idx / 8, c = idx % 8;
      *(uint2 *)(sv + d * VROW + c * 16) = make_uint2(rv[i].x, rv[i].y);
      *(uint2 *)(sv + d * VROW + c * 16 + 8) = make_uint2(rv[i].z, rv[i].w);
    }
  };

  floatx16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = 1.4426950408889634f * rsqrtf((float)HD);   // log2(e) / sqrt(hd)
  const float inv_sc = 1.0f / sc;

  long long t_begin = 0, t_wait = 0, t_pro = 0;
  if constexpr (PROF) t_begin = clock64();
  load_tile(0);
  store_tile(0);
  __syncthreads();
  if constexpr (PROF) t_pro = clock64() - t_begin;
  for (int t = 0; t < n_tiles; ++t) {
    if (t + 1 < n_tiles) load_tile(t + 1);
    const int key0 = t * BKV;
    if (key0 <= wave_last) {   // wave-uniform: tiles entirely above the diagonal are skipped
      const unsigned char *sk = smem + (t & 1) * STAGE;
      const unsigned char *sv = sk + K_BYTES;
      floatx16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
      // K operand fragments are fetched one group (GK MFMAs' worth) ahead of their use, and the
      // first V^T fragments are requested before the softmax arithmetic starts.
      constexpr int NG = DS / 2;              // groups per tile: two d steps x two key blocks = 4 independent-ish MFMAs
      bf16x8 kfr[2][4];
      uint4 vfr[2][DB];
      auto load_k = [&](int buf, int gi) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int kb = i & 1, ds = gi * 2 + (i >> 1);
          kfr[buf][i] = *(const bf16x8 *)(sk + (kb * 32 + l32) * KROW + (ds * 2 + g) * 16);
        }
      };
      auto load_v = [&](int buf, int st) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const unsigned char *vp = sv + (db * 32 + l32) * VROW + (st * 16 + 4 * g) * 2;
          uint2 lo = *(const uint2 *)vp, hi = *(const uint2 *)(vp + 16);
          vfr[buf][db] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
      };
      load_k(0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int gi = 0; gi < NG; ++gi) {
        if (gi + 1 < NG) load_k((gi + 1) & 1, gi + 1); else load_v(0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {   // alternate the two accumulators so consecutive MFMAs are independent
          const int kb = i & 1, ds = gi * 2 + (i >> 1);
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[gi & 1][i], qf[ds], s[kb], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // s[kb][4*jg+e] = raw score(key = key0 + kb*32 + 8*jg + 4*g + e, this lane's query)
      const bool need_mask = (key0 + BKV - 1 > qb.q0 + wave * 32) || (key0 + BKV > qb.n);
      if (need_mask) {   // wave-uniform: only tiles on the diagonal or at the end of the sequence
        // element (kb, v) is key key0 + 4*g + kb*32 + 8*(v>>2) + (v&3); visible iff key <= min(qpos, n-1)
        const int lim = (qpos < qb.n - 1 ? qpos : qb.n - 1) - key0 - 4 * g;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][v] = (kb * 32 + 8 * (v >> 2) + (v & 3) > lim) ? -INFINITY : s[kb][v];
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = __builtin_fmaxf(mx, s[kb][v]);
      mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
      // Lazy rescaling: the reference maximum m_run (raw score units) only moves when some query's
      // tile maximum exceeds it by more than 8/sc, i.e. when an exponential would exceed 2^8.  The
      // result is unchanged (numerator and denominator share m_run); the 64-register rescale of O
      // is skipped on most tiles.  Every query sees key 0 in tile 0, so m_run is finite from then on.
      if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f * inv_sc) != 0) {
        const float m_new = __builtin_fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
      }
      const float msc = m_run * sc;
      float rs = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], sc, -msc));   // exp2 of (-inf) is 0
          s[kb][v] = e;
          rs += e;
        }
      l_run += rs;
      // O^T += V^T P^T, 16 keys per MFMA: step st uses s[st/2][(st%2)*8 .. +8]
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s[st >> 1][(st & 1) * 8 + e];
        if (st + 1 < 4) load_v((st + 1) & 1, st + 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < DB; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfr[st & 1][db]), pf, o[db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    long long tw0 = 0;
    if constexpr (PROF) tw0 = clock64();
    if (t + 1 < n_tiles) store_tile((t + 1) & 1);
    __syncthreads();
    if constexpr (PROF) t_wait += clock64() - tw0;
  }
  if constexpr (PROF) {
    if (lane == 0 && p.prof) {
      long long *o4 = p.prof + ((long long)(blockIdx.y * gridDim.x + blockIdx.x) * 4 + wave) * 4;
      o4[0] = clock64() - t_begin; o4[1] = t_wait; o4[2] = t_pro; o4[3] = n_tiles;
    }
  }

  // ---- normalise and store: o[db][4*jg+e] = O[query][d = db*32 + 8*jg + 4*g + e] ----
  float l_tot = l_run + __shfl_xor(l_run, 32);
  if (!qvalid) return;
  const float inv = 1.f / l_tot;
  bf16_t *op = p.out + (int64_t)qrow * q_dim + head * HD;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int jg = 0; jg < 4; ++jg) {
      *(uint2 *)(op + db * 32 + 8 * jg + 4 * g) =
          make_uint2(pack_bf16x2(o[db][4 * jg] * inv, o[db][4 * jg + 1] * inv), pack_bf16x2(o[db][4 * jg + 2] * inv, o[db][4 * jg + 3] * inv));
    }
}

// --------------------------------------------------------------- decode ----
// grid (n_rows, n_kv_heads, n_split); 256 threads.  Each group of LPK lanes
// (hd/8) owns one key at a time and 8 dims of it; the R = Hq/Hkv query heads of
// the KV head are processed together so K/V bytes are read once.
template <int HD, int R>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnDecodeParams p) {
  constexpr int LPK = HD / 8;           // lanes per key
  constexpr int KPW = 64 / LPK;         // keys per wave per step
  constexpr int KPS = KPW * 4;          // keys per workgroup step
  const DecodeRow row = p.rows[blockIdx.x];
  const int kvh = blockIdx.y, split = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPK, grp = lane / LPK;
  const int q_dim = p.n_q_heads * HD;
  const int kv_dim = p.n_kv_heads * HD;

  // keys of this split
  const int per = (row.n_keys + p.n_split - 1) / p.n_split;
  const int k_lo = split * per;
  const int k_hi = (k_lo + per) < row.n_keys ? (k_lo + per) : row.n_keys;

  // query fragments (8 dims of each of the R heads), rotated here if asked
  float q[R][8];
  const float sc = 1.4426950408889634f * rsqrtf((float)HD);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bf16_t *qp = p.q + (int64_t)row.q_row * q_dim + (kvh * R + r) * HD;
    uint4 u = *(const uint4 *)(qp + sub * 8);
    float x[8] = {bf16lo(u.x), bf16hi(u.x), bf16lo(u.y), bf16hi(u.y), bf16lo(u.z), bf16hi(u.z), bf16lo(u.w), bf16hi(u.w)};
    if (row.cs_row >= 0) {
      const int psub = (sub + LPK / 2) % LPK;   // chunk holding the rotary partners
      uint4 w = *(const uint4 *)(qp + psub * 8);
      float y[8] = {bf16lo(w.x), bf16hi(w.x), bf16lo(w.y), bf16hi(w.y), bf16lo(w.z), bf16hi(w.z), bf16lo(w.w), bf16hi(w.w)};
      const bool first = sub < LPK / 2;
      const float2 *cs = p.cos_sin + (int64_t)row.cs_row * (HD / 2) + (first ? sub : psub) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float2 c = cs[e];
        // first half: x*cos - partner*sin ; second half: x*cos + partner*sin
        float v = first ? (x[e] * c.x - y[e] * c.y) : (x[e] * c.x + y[e] * c.y);
        x[e] = bf16_to_f32(f32_to_bf16(v));   // q is held in bf16 like the prefill path's
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) q[r][e] = x[e] * sc;
  }

  float m[R], l[R], acc[R][8];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    m[r] = -INFINITY; l[r] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
  }
  const float ks = p.fp8 ? p.scale_k[kvh] : 1.f, vs = p.fp8 ? p.scale_v[kvh] : 1.f;
  const int32_t *bt = p.block_tables + (int64_t)row.seq * p.max_blocks_per_seq;

  for (int kb = k_lo + wave * KPW; kb < k_hi; kb += KPS) {
    const int key = kb + grp;
    const bool valid = key < k_hi;
    float kf[8], vf[8];
    if (valid) {
      int blk = bt[key / SKV_BLOCK];
      blk = ((unsigned)blk < (unsigned)p.n_blocks) ? blk : 0;   // bad ids are flagged by the plan kernel; never dereference them
      const int64_t slot = (int64_t)blk * SKV_BLOCK + key % SKV_BLOCK;
      const int64_t off = (slot * p.n_kv_heads + kvh) * HD + sub * 8;
      if (p.fp8) {
        uint2 kc = *(const uint2 *)((const uint8_t *)p.cache_k + off);
        uint2 vc = *(const uint2 *)((const uint8_t *)p.cache_v + off);
        uint32_t kw[2] = {kc.x, kc.y}, vw[2] = {vc.x, vc.y};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          kf[e] = e4m3fn_to_f32((uint8_t)(kw[e >> 2] >> ((e & 3) * 8))) * ks;
          vf[e] = e4m3fn_to_f32((uint8_t)(vw[e >> 2] >> ((e & 3) * 8))) * vs;
        }
      } else {
        uint4 ku = *(const uint4 *)((const bf16_t *)p.cache_k + off);
        uint4 vu = *(const uint4 *)((const bf16_t *)p.cache_v + off);
        kf[0] = bf16lo(ku.x); kf[1] = bf16hi(ku.x); kf[2] = bf16lo(ku.y); kf[3] = bf16hi(ku.y);
        kf[4] = bf16lo(ku.z); kf[5] = bf16hi(ku.z); kf[6] = bf16lo(ku.w); kf[7] = bf16hi(ku.w);
        vf[0] = bf16lo(vu.x); vf[1] = bf16hi(vu.x); vf[2] = bf16lo(vu.y); vf[3] = bf16hi(vu.y);
        vf[4] = bf16lo(vu.z); vf[5] = bf16hi(vu.z); vf[6] = bf16lo(vu.w); vf[7] = bf16hi(vu.w);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) { kf[e] = 0.f; vf[e] = 0.f; }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d += q[r][e] * kf[e];
#pragma unroll
      for (int o = LPK / 2; o > 0; o >>= 1) d += __shfl_xor(d, o);
      if (!valid) d = -INFINITY;
      const float mn = fmaxf(m[r], d);
      if (mn != -INFINITY) {
        const float a = exp2f(m[r] - mn), w = exp2f(d - mn);
        l[r] = l[r] * a + w;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = acc[r][e] * a + w * vf[e];
        m[r] = mn;
      }
    }
  }

  // ---- combine the key groups of a wave (lanes with equal `sub`), then the waves ----
  __shared__ float sm[4][R][HD + 2];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float mw = m[r];
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
    const float a = (m[r] == -INFINITY) ? 0.f : exp2f(m[r] - mw);
    float lw = l[r] * a;
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) lw += __shfl_xor(lw, o);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = acc[r][e] * a;
#pragma unroll
      for (int o = LPK; o < 64; o <<= 1) x += __shfl_xor(x, o);
      if (grp == 0) sm[wave][r][sub * 8 + e] = x;
    }
    if (lane == 0) { sm[wave][r][HD] = mw; sm[wave][r][HD + 1] = lw; }
  }
  __syncthreads();
  for (int i = tid; i < R * HD; i += 256) {
    const int r = i / HD, d = i % HD;
    float mm = fmaxf(fmaxf(sm[0][r][HD], sm[1][r][HD]), fmaxf(sm[2][r][HD], sm[3][r][HD]));
    float x = 0.f, ll = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = sm[w][r][HD];
      const float a = (mw == -INFINITY) ? 0.f : exp2f(mw - mm);
      x += a * sm[w][r][d];
      ll += a * sm[w][r][HD + 1];
    }
    float *dst = p.partial + (((int64_t)blockIdx.x * p.n_q_heads + kvh * R + r) * p.n_split + split) * (HD + 2);
    dst[d] = x;
    if (d == 0) { dst[HD] = mm; dst[HD + 1] = ll; }
  }
}

}  // namespace

int launch_attention_prefill(const AttnPrefillParams &p, hipStream_t st) {
  if (p.n_qblocks <= 0) return 0;
  dim3 grid(p.n_qblocks, p.n_q_heads);
  if (p.head_dim == 128) {
    constexpr int SMEM = 2 * (BKV * (128 * 2 + 16) + 128 * (BKV * 2 + 8));
    static bool set = false;
    if (!set) {
      hipError_t e = hipFuncSetAttribute((const void *)attn_prefill_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
      if (e != hipSuccess) return (int)e;
      set = true;
    }
    if (p.prof) {
      (void)hipFuncSetAttribute((const void *)attn_prefill_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
      hipLaunchKernelGGL((attn_prefill_kernel<128, true>), grid, dim3(256), SMEM, st, p);
      return 0;
    }
    hipLaunchKernelGGL(attn_prefill_kernel<128>, grid, dim3(256), SMEM, st, p);
  } else {
    constexpr int SMEM = 2 * (BKV * (64 * 2 + 16) + 64 * (BKV * 2 + 8));
    hipLaunchKernelGGL(attn_prefill_kernel<64>, grid, dim3(256), SMEM, st, p);
  }
  return 0;
}

template <int HD>
static int launch_decode_hd(const AttnDecodeParams &p, hipStream_t st) {
  dim3 grid(p.n_rows, p.n_kv_heads, p.n_split);
  const int R = p.n_q_heads / p.n_kv_heads;
  switch (R) {
    case 1: hipLaunchKernelGGL((attn_decode_kernel<HD, 1>), grid, dim3(256), 0, st, p); break;
    case 2: hipLaunchKernelGGL((attn_decode_kernel<HD, 2>), grid, dim3(256), 0, st, p); break;
    case 4: hipLaunchKernelGGL((attn_decode_kernel<HD, 4>), grid, dim3(256), 0, st, p); break;
    case 8: hipLaunchKernelGGL((attn_decode_kernel<HD, 8>), grid, dim3(256), 0, st, p); break;
    default: return -1;
  }
  return 0;
}
int launch_attention_decode(const AttnDecodeParams &p, hipStream_t st) {
  if (p.n_rows <= 0) return 0;
  return p.head_dim == 128 ? launch_decode_hd<128>(p, st) : launch_decode_hd<64>(p, st);
}
