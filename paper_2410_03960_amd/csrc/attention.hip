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
// 2. attn_decode_kernel: one query row against a paged bf16 cache, split over key
//    ranges; used for the last-token tail and for decode tokens.
// 3. attn_decode_fp8_kernel: the same over an e4m3 cache, the codes fed to the
//    matrix unit as they are.
#include "common.h"

namespace {

constexpr int BQ = 128;   // queries per workgroup
constexpr int BKV = 64;   // keys per tile

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_addr + 16*i
// (M0 carries the LDS base).  The waits are placed by hand (s_waitcnt vmcnt) because the
// compiler cannot tell which LDS bytes a request targets.
__device__ __forceinline__ void lds_dma16(const void *gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}

// max(x[lane], x[lane ^ 32]) without going through LDS: v_permlane32_swap exchanges the upper half
// of its first operand with the lower half of its second, leaving (lo, lo) and (hi, hi).
__device__ __forceinline__ float cross_half_max(float x) {
  unsigned a = __builtin_bit_cast(unsigned, x), b = a;
  asm volatile("" : "+v"(b));   // two distinct registers
  auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  return __builtin_fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}

// LDS tiles are unpadded and filled by LDS-DMA in 1 KB pieces; 16-byte chunks are XOR-swizzled
// inside a row so that the 16 lanes served per LDS cycle (256 bytes, 64 banks) never collide:
//   K   tile [64 keys][HD*2 bytes]:  chunk c of row r sits at c ^ swz_k(r)
//   V^T tile [HD dims][128 bytes]:   chunk c of row d sits at c ^ ((d >> 1) & 7)
// The 32 MFMA rows of a key block are fed with the keys in the order bit2 <-> bit3 swapped, which
// makes the 8 exponentials a lane holds per PV step belong to 8 consecutive keys -- one 16-byte
// V^T chunk instead of two 8-byte halves.
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(AttnPrefillParams p) {
  constexpr int KCH = HD / 8;              // 16-byte chunks per K row (16 or 8)
  constexpr int K_RPI = 64 / KCH;          // K rows per 1 KB DMA request (4 or 8)
  constexpr int K_BYTES = BKV * HD * 2, V_BYTES = HD * BKV * 2;
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int K_IT = K_BYTES / 1024 / 4; // DMA requests per wave per K tile
  constexpr int V_IT = V_BYTES / 1024 / 4; // ... per V^T tile (8 rows of 128 bytes each)
  constexpr int DS = HD / 16;              // d steps of the QK^T contraction
  constexpr int DB = HD / 32;              // 32-wide d blocks of the output

  extern __shared__ __align__(16) unsigned char smem[];

  // Persistent workgroups pull items from device counters.  Item = (query block, head), query
  // blocks sorted longest first by the plan, so the long items start first and the short ones fill
  // the end; the next item is requested while the current one is being computed.
  // Workgroup w runs on XCD w mod 8, each XCD with its own L2.  With a multiple of 8 query heads
  // there is one queue per XCD holding the head slots == XCD (mod 8), and head slot s stands for
  // head (s mod Hkv) * (Hq / Hkv) + s / Hkv: the query heads that share a KV head meet in one L2.
  __shared__ int s_item;
  const int NQ = (p.n_q_heads % 8 == 0) ? 8 : 1;
  const int qid = blockIdx.x % NQ, hpq = p.n_q_heads / NQ;
  const int n_items = p.n_qblocks * hpq;   // per queue
  if (threadIdx.x == 0) s_item = atomicAdd(p.sched + qid, 1);
  __syncthreads();
  for (;;) {
  const int item = s_item;
  if (item >= n_items) break;
  int item_next = 0;
  if (threadIdx.x == 0) item_next = atomicAdd(p.sched + qid, 1);   // consumed after the last tile
  const int qblock = item / hpq;
  const QBlock qb = p.qblocks[qblock];
  const int hslot = (item % hpq) * NQ + qid;
  const int kvh = hslot % p.n_kv_heads;
  const int head = kvh * (p.n_q_heads / p.n_kv_heads) + hslot / p.n_kv_heads;
  const int q_dim = p.n_q_heads * HD, kv_dim = p.n_kv_heads * HD;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;

  // ---- this lane's query: position and Q fragments (second MFMA operand) ----
  const int qpos = qb.q0 + wave * 32 + l32;            // position in the sequence
  const bool qvalid = qpos < qb.n;
  const int qrow = qb.row0 + wave * 32 + l32;
  const int qrow_c = qvalid ? qrow : qb.q_last_row;
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

  typedef __attribute__((address_space(3))) void *lds_ptr_t;
  const unsigned lds_base = (unsigned)(size_t)(lds_ptr_t)smem;

  // ---- DMA sources of this lane ----
  // K request i of this wave covers rows (wave*K_IT + i)*K_RPI ... of the tile; this lane fetches
  // row k_r0 + i*K_RPI, chunk k_c0 ^ 4i (the swizzle, folded: wave*K_IT*K_RPI is a multiple of 16).
  // V^T request i covers dims (wave*V_IT + i)*8 ...; chunk v_c0 ^ 4*(i&1).
  const int k_r0 = wave * K_IT * K_RPI + lane / KCH;
  const int k_c0 = (lane % KCH) ^ (HD == 128 ? (lane >> 4) : (lane >> 4));
  const int v_d0 = wave * V_IT * 8 + (lane >> 3);
  const int v_c0 = (lane & 7) ^ (lane >> 4);
  const bf16_t *v_src0 = vbase + (int64_t)v_d0 * p.vt_ld + v_c0 * 8;
  const bf16_t *v_src1 = vbase + (int64_t)v_d0 * p.vt_ld + (v_c0 ^ 4) * 8;
  // request idx (0 .. K_IT+V_IT-1) of tile t into `stage`: the K rows first, then the V^T rows
  auto issue_one = [&](int idx, int t, int stage) {
    const int key0 = t * BKV;
    const unsigned st = lds_base + stage * STAGE;
#pragma unroll
    for (int i = 0; i < K_IT; ++i)
      if (idx == i) {
        int key = key0 + k_r0 + i * K_RPI;
        key = key < qb.n ? key : qb.n - 1;   // rows past the end are masked later; any finite data will do
        lds_dma16(kbase + ((int64_t)key * kv_dim + ((k_c0 ^ (4 * i)) * 8)), st + (wave * K_IT + i) * 1024);
      }
#pragma unroll
    for (int i = 0; i < V_IT; ++i)
      if (idx == K_IT + i)   // padded columns are zero
        lds_dma16(((i & 1) ? v_src1 : v_src0) + ((int64_t)(8 * i) * p.vt_ld + key0), st + K_BYTES + (wave * V_IT + i) * 1024);
  };
  auto issue_tile = [&](int t, int stage) {
#pragma unroll
    for (int i = 0; i < K_IT + V_IT; ++i) issue_one(i, t, stage);
  };

  // ---- LDS read addresses of this lane ----
  // K operand: MFMA row l32 of key block kb is key kb*32 + swap23(l32); both blocks share the swizzle.
  // Chunk (2*ds + g) ^ swz = (2*ds) ^ (g ^ swz): the d step enters as one XOR of the byte address with
  // 32*ds (the chunk bits of the row bases are zero), likewise the PV step for V^T.
  const int krow = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
  const unsigned k_lane = krow * (HD * 2) + ((g ^ (HD == 128 ? (krow & 15) : ((krow >> 1) & 7))) << 4);
  // V^T operand: dims db*32 + l32; all d blocks share the swizzle
  const unsigned v_lane = K_BYTES + l32 * 128 + ((g ^ ((l32 >> 1) & 7)) << 4);

  floatx16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = 1.4426950408889634f * rsqrtf((float)HD);   // log2(e) / sqrt(hd)
  const float inv_sc = 1.0f / sc;

  issue_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();
  for (int t = 0; t < n_tiles; ++t) {
    asm volatile("" ::: "memory");
    // Tile t+1 goes into the stage every wave finished reading before the last barrier.  The requests
    // are spread over the MFMA phases (a burst would hold the wave at the address unit's queue).
    // After the last tile the requests simply repeat it into the idle stage (no branches in the phases).
    const int tn = t + 1 < n_tiles ? t + 1 : t, sn = (t + 1) & 1;
    const int key0 = t * BKV;
    if (key0 > wave_last) issue_tile(tn, sn);
    asm volatile("" ::: "memory");
    if (key0 <= wave_last) {   // wave-uniform: tiles entirely above the diagonal are skipped
      const unsigned k_addr = (t & 1) * STAGE + k_lane, v_addr = (t & 1) * STAGE + v_lane;
      floatx16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
      // K operand fragments are fetched one d step ahead of their use (the SIMD's other wave covers
      // the rest of the LDS latency), and the first V^T fragments before the softmax arithmetic starts.
      bf16x8 kfr[2][2];                       // two d steps (both key blocks each)
      bf16x8 vfr[DB];
      auto load_k = [&](int ds) {
        const unsigned char *kp = smem + (k_addr ^ (unsigned)(ds * 32));
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kfr[ds % 2][kb] = *(const bf16x8 *)(kp + kb * (32 * HD * 2));
      };
      auto load_v = [&](int st, int db) {   // keys 16*st + 8*g .. +7 of dim db*32 + l32
        vfr[db] = *(const bf16x8 *)(smem + (v_addr ^ (unsigned)(st * 32)) + db * 4096);
      };
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_setprio(2);   // the MFMA phases win the issue arbitration against the other wave's softmax arithmetic
      load_k(0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) {
        if (ds + 1 < DS) load_k(ds + 1);
        else {
#pragma unroll
          for (int db = 0; db < DB; ++db) load_v(0, db);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)   // the two accumulators alternate, so consecutive MFMAs are independent
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ds % 2][kb], qf[ds], s[kb], 0, 0, 0);
        static_assert(K_IT + V_IT == DS, "one request of the next tile per d step");
        issue_one(ds, tn, sn);   // all of the next tile is requested in this phase: the K rows first, then the V^T rows
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_s_setprio(0);
      __builtin_amdgcn_sched_barrier(0);   // phase boundaries keep the scheduler from stretching live ranges across phases
      asm volatile("" ::: "memory");
      // s[kb][v] = raw score(key = key0 + kb*32 + 16*(v>>3) + 8*g + (v&7), this lane's query)
      const bool need_mask = (key0 + BKV - 1 > qb.q0 + wave * 32) || (key0 + BKV > qb.n);
      if (need_mask) {   // wave-uniform: only tiles on the diagonal or at the end of the sequence
        // visible iff key <= min(qpos, n-1)
        const int lim = (qpos < qb.n - 1 ? qpos : qb.n - 1) - key0 - 8 * g;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][v] = (kb * 32 + 16 * (v >> 3) + (v & 7) > lim) ? -INFINITY : s[kb][v];
      }
      // (four independent chains: a lone wave issues dependent vector instructions well below full rate)
      float mx4[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx4[(kb * 16 + v) / 8] = __builtin_fmaxf(mx4[(kb * 16 + v) / 8], s[kb][v]);
      float mx = __builtin_fmaxf(__builtin_fmaxf(mx4[0], mx4[1]), __builtin_fmaxf(mx4[2], mx4[3]));
      mx = cross_half_max(mx);   // (a shuffle through LDS would also wait for the V^T fragments just requested)
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
      float rs4[4] = {0.f, 0.f, 0.f, 0.f};   // row sum in four independent chains (by PV step), added up in a fixed order
      // exponentials of PV step st (keys 16*st + 8*g .. +7), two at a time, straight into the bf16 operand
      bf16x8 pf[2];
      auto exp_pair = [&](int st, int j) {
#pragma unroll
        for (int e = 2 * j; e < 2 * j + 2; ++e) {
          const float x = __builtin_amdgcn_exp2f(__builtin_fmaf(s[st >> 1][(st & 1) * 8 + e], sc, -msc));   // exp2 of (-inf) is 0
          rs4[st] += x;
          pf[st & 1][e] = (__bf16)x;
        }
      };
#pragma unroll
      for (int j = 0; j < 4; ++j) exp_pair(0, j);
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_setprio(1);
      // O^T += V^T P^T, 16 keys per MFMA.  The exponentials of the next step are computed between
      // the MFMAs of this one, and each V^T fragment register is refilled right after its use.
#pragma unroll
      for (int st = 0; st < 4; ++st) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[db], pf[st & 1], o[db], 0, 0, 0);
          if (st + 1 < 4) {
            load_v(st + 1, db);
            if (DB == 4) exp_pair(st + 1, db);
            else { exp_pair(st + 1, 2 * db); exp_pair(st + 1, 2 * db + 1); }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      l_run += (rs4[0] + rs4[1]) + (rs4[2] + rs4[3]);
      __builtin_amdgcn_s_setprio(0);
      asm volatile("" ::: "memory");
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);   // this wave's part of tile t+1 has landed ...
    __syncthreads();                      // ... everyone's has, and everyone is done reading tile t
  }

  // ---- normalise and store: o[db][4*jg+e] = O[query l32][d = db*32 + 8*jg + 4*g + e] ----
  // The wave's 32 x HD block leaves through LDS, so that it is written as whole rows (16 lanes cover
  // one 256-byte row); stored straight from the accumulator layout it went out as 16-byte pieces of
  // 32 rows per instruction, which cost a third of the kernel's time on short sequences.  The slab is
  // this wave's 8 KB of the second stage: every wave is past the last tile's barrier, and the next
  // requests into that stage follow the next item's first barrier.  16-byte chunks are XOR-swizzled
  // by the row.
  {
    const float inv = 1.f / (l_run + __shfl_xor(l_run, 32));
    unsigned char *slab = smem + STAGE + wave * (32 * HD * 2);
    unsigned char *wrow = slab + l32 * (HD * 2);
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int jg = 0; jg < 4; ++jg)
        *(uint2 *)(wrow + (((db * 4 + jg) ^ (l32 & (KCH - 1))) << 4) + 8 * g) =
            make_uint2(pack_bf16x2(o[db][4 * jg] * inv, o[db][4 * jg + 1] * inv), pack_bf16x2(o[db][4 * jg + 2] * inv, o[db][4 * jg + 3] * inv));
    // a wave's LDS operations execute in order: the reads below see the writes above
    const int c = lane % KCH, r0 = lane / KCH;
    // row j*K_RPI + r0: its swizzle is r0 | (j*K_RPI mod KCH) (disjoint bits), so j enters as an XOR with a constant
    const unsigned roff = r0 * (HD * 2) + ((c ^ r0) << 4);
    bf16_t *op = p.out + ((int64_t)(qb.row0 + wave * 32 + r0) * q_dim + head * HD + c * 8);
    const int rows_left = qb.n - (qb.q0 + wave * 32) - r0;   // row j*K_RPI + r0 exists iff j*K_RPI < rows_left
#pragma unroll
    for (int j = 0; j < 32 / K_RPI; ++j) {
      const int jr = j * K_RPI;
      const uint4 val = *(const uint4 *)(slab + ((roff + jr * (HD * 2)) ^ (unsigned)((jr & (KCH - 1)) << 4)));
      if (jr < rows_left) *(uint4 *)(op + (int64_t)jr * q_dim) = val;
    }
  }
  // every wave read s_item before the tile loop's barriers; the same barriers separate the last
  // tile's LDS reads from the next prologue's writes
  if (threadIdx.x == 0) s_item = item_next;
  __syncthreads();
  }
  // the last workgroup to leave zeroes the counters for the next launch
  if (threadIdx.x == 0) {
    __threadfence();
    if (atomicAdd(p.sched + 8, 1) == (int)gridDim.x - 1) {
      for (int i = 0; i < 9; ++i) p.sched[i] = 0;
      __threadfence();
    }
  }
}

// Sum over the LPK (8 or 16) consecutive lanes that share a key, result in all of them: data-parallel
// primitives inside a row of 16 lanes (quad swaps, mirror of 8, mirror of 16), no LDS round trip.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
template <int LPK>
__device__ __forceinline__ float key_group_sum(float x) {
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);   // row_half_mirror: lane i <-> 7 - i of each 8
  if constexpr (LPK == 16) x = dpp_add<0x140>(x);   // row_mirror: lane i <-> 15 - i
  return x;
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
  // at least 128 keys per split (four iterations of the loop below): a row much shorter than the batch's
  // longest uses fewer splits (the rest see an empty range and report a weight of zero)
  int per = (row.n_keys + p.n_split - 1) / p.n_split;
  per = per < 128 ? 128 : per;
  const int k_lo = split * per;
  const int k_hi = (k_lo + per) < row.n_keys ? (k_lo + per) : row.n_keys;

  // query fragments (8 dims of each of the R heads), rotated here if asked; kept as the four bf16 pairs
  // they are stored as, for the two-element bf16 dot product (the score scale is applied to the sum)
  uint32_t q[R][4];
  const float sc = 1.4426950408889634f * rsqrtf((float)HD);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bf16_t *qp = p.q + (int64_t)row.q_row * q_dim + (kvh * R + r) * HD;
    uint4 u = *(const uint4 *)(qp + sub * 8);
    if (row.cs_row >= 0) {
      float x[8] = {bf16lo(u.x), bf16hi(u.x), bf16lo(u.y), bf16hi(u.y), bf16lo(u.z), bf16hi(u.z), bf16lo(u.w), bf16hi(u.w)};
      const int psub = (sub + LPK / 2) % LPK;   // chunk holding the rotary partners
      uint4 w = *(const uint4 *)(qp + psub * 8);
      float y[8] = {bf16lo(w.x), bf16hi(w.x), bf16lo(w.y), bf16hi(w.y), bf16lo(w.z), bf16hi(w.z), bf16lo(w.w), bf16hi(w.w)};
      const bool first = sub < LPK / 2;
      const float2 *cs = p.cos_sin + (int64_t)row.cs_row * (HD / 2) + (first ? sub : psub) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float2 c = cs[e];
        // first half: x*cos - partner*sin ; second half: x*cos + partner*sin
        x[e] = first ? (x[e] * c.x - y[e] * c.y) : (x[e] * c.x + y[e] * c.y);
      }
      // q is held in bf16 like the prefill path's
      u = make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7]));
    }
    q[r][0] = u.x; q[r][1] = u.y; q[r][2] = u.z; q[r][3] = u.w;
  }

  float m[R], l[R], acc[R][8];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    m[r] = -INFINITY; l[r] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
  }
  const int32_t *bt = p.block_tables + (int64_t)row.seq * p.max_blocks_per_seq;

  // Two key steps per iteration, all four loads first.  The running reference m[r] (log2 units) only
  // moves when a score exceeds it by more than 8, so most keys cost one exponential and no rescale of
  // the accumulators; numerator and denominator share the reference, the result is unchanged.
  // The block ids of the next iteration's keys are looked up one iteration ahead, so that a K/V load
  // does not wait for a table lookup first (keys past the end read the entry of the last key).
  int blk_nxt[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int key = k_lo + wave * KPW + u * KPS + grp;
    blk_nxt[u] = k_hi > 0 ? bt[(key < k_hi ? key : k_hi - 1) / SKV_BLOCK] : 0;
  }
  for (int kb = k_lo + wave * KPW; kb < k_hi; kb += 2 * KPS) {
    float vf[2][8];
    bool valid[2];
    uint4 kraw[2], vraw[2];
    const int blk_cur[2] = {blk_nxt[0], blk_nxt[1]};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int key = kb + 2 * KPS + u * KPS + grp;
      blk_nxt[u] = bt[(key < k_hi ? key : k_hi - 1) / SKV_BLOCK];
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int key = kb + u * KPS + grp;
      valid[u] = key < k_hi;
      kraw[u] = make_uint4(0, 0, 0, 0); vraw[u] = make_uint4(0, 0, 0, 0);
      if (valid[u]) {
        int blk = blk_cur[u];
        blk = ((unsigned)blk < (unsigned)p.n_blocks) ? blk : 0;   // bad ids are flagged by the plan kernel; never dereference them
        const int64_t slot = (int64_t)blk * SKV_BLOCK + key % SKV_BLOCK;
        const int64_t off = (slot * p.n_kv_heads + kvh) * HD + sub * 8;
        kraw[u] = *(const uint4 *)((const bf16_t *)p.cache_k + off);
        vraw[u] = *(const uint4 *)((const bf16_t *)p.cache_v + off);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const uint32_t kw[4] = {kraw[u].x, kraw[u].y, kraw[u].z, kraw[u].w}, vw[4] = {vraw[u].x, vraw[u].y, vraw[u].z, vraw[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) { vf[u][2 * e] = bf16lo(vw[e]); vf[u][2 * e + 1] = bf16hi(vw[e]); }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kw[e]), __builtin_bit_cast(bf16x2_t, q[r][e]), d, false);
        d = key_group_sum<LPK>(d) * sc;
        if (valid[u] && d > m[r] + 8.0f) {   // uniform within the key's lanes
          const float a = __builtin_amdgcn_exp2f(m[r] - d);   // exp2(-inf) = 0 the first time
          l[r] *= a;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[r][e] *= a;
          m[r] = d;
        }
        const float w = valid[u] ? __builtin_amdgcn_exp2f(d - m[r]) : 0.f;
        l[r] += w;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] += w * vf[u][e];
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

// ------------------------------------------------ decode, FP8 cache, MFMA ----
// Single-query attention over an e4m3 cache with the codes fed to the matrix unit as they are
// (v_mfma_f32_16x16x32_fp8_fp8), scales applied to the fp32 results.  grid (n_rows, n_kv_heads, n_split),
// 4 waves, each wave walks 32 keys per step.
//  * S^T[key][r] = sum_d K[key][d] q[r][d]: first operand = K codes straight from the cache (a lane reads
//    HD/4 contiguous bytes of one key; within one instruction the contraction index may be assigned to
//    (lane group, element) in any order as long as both operands agree), second operand = the R query heads
//    of the KV head (columns R..15 are zero) as e4m3 with one scale per head.  To keep bf16-level accuracy q
//    is split into two e4m3 terms, q = qs * (q_hi + q_lo), each with its own instruction.
//  * O^T[d][r] += sum_key V^T[d][key] P^T[key][r]: V codes are staged row-major in LDS and read with the
//    transposing LDS read (ds_read_b64_tr_b8: lane i of a 16-lane group receives column i of the 8 x 16 byte
//    matrix the group's lanes address), which yields the [d][8 keys] fragments without any byte shuffles;
//    the softmax weights are the second operand, again as two e4m3 terms.
// The 32 keys of a step sit in the contraction slots in the order the score instruction leaves them:
// slot (g, j) of lane group g holds key 4g + j for j < 4 and key 16 + 4g + (j - 4) for j >= 4.
typedef long fp8x8_t;   // eight e4m3 codes
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int pack4_fp8(float a, float b, float c, float d) {
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
  return __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
}
__device__ __forceinline__ fp8x8_t make_fp8x8(int lo, int hi) {
  return (fp8x8_t)(((unsigned long)(unsigned)hi << 32) | (unsigned long)(unsigned)lo);
}
// x[0..7] -> e4m3 term `hi` and e4m3 term `lo` of the remainder
__device__ __forceinline__ void split_fp8x8(const float (&x)[8], fp8x8_t &hi, fp8x8_t &lo) {
  const int h0 = pack4_fp8(x[0], x[1], x[2], x[3]), h1 = pack4_fp8(x[4], x[5], x[6], x[7]);
  float r[8];
  r[0] = x[0] - __builtin_amdgcn_cvt_f32_fp8(h0, 0); r[1] = x[1] - __builtin_amdgcn_cvt_f32_fp8(h0, 1);
  r[2] = x[2] - __builtin_amdgcn_cvt_f32_fp8(h0, 2); r[3] = x[3] - __builtin_amdgcn_cvt_f32_fp8(h0, 3);
  r[4] = x[4] - __builtin_amdgcn_cvt_f32_fp8(h1, 0); r[5] = x[5] - __builtin_amdgcn_cvt_f32_fp8(h1, 1);
  r[6] = x[6] - __builtin_amdgcn_cvt_f32_fp8(h1, 2); r[7] = x[7] - __builtin_amdgcn_cvt_f32_fp8(h1, 3);
  hi = make_fp8x8(h0, h1);
  lo = make_fp8x8(pack4_fp8(r[0], r[1], r[2], r[3]), pack4_fp8(r[4], r[5], r[6], r[7]));
}

template <int HD, int R>
__global__ __launch_bounds__(256) void attn_decode_fp8_kernel(AttnDecodeParams p) {
  constexpr int NM = HD / 32;        // score instructions per 16-key block and q term
  constexpr int NDB = HD / 16;       // 16-dim blocks of the output
  constexpr int VS = HD + 16;        // LDS row stride of the V tile (keeps the transposing reads off shared banks)
  constexpr int KB = HD / 4;         // contiguous K bytes a lane reads per key
  constexpr int VCH = HD / 16;       // 16-byte chunks per V row
  constexpr int V_IT = 32 * VCH / 64;  // 16-byte loads per lane for a 32-key V tile
  __shared__ __align__(16) unsigned char v_lds[4][32 * VS];
  __shared__ __align__(16) float q32[R][HD];
  __shared__ __align__(16) unsigned char q8[2][16][HD];
  __shared__ float q_scale[8];
  __shared__ float sm[4][R][HD + 2];

  const DecodeRow row = p.rows[blockIdx.x];
  const int kvh = blockIdx.y, split = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, kq = lane >> 4;
  const int q_dim = p.n_q_heads * HD;
  const bool per_slot = p.fp8 == 2;

  // keys of this split: whole 128-key steps, at least 256 keys per split
  int per = (row.n_keys + p.n_split - 1) / p.n_split;
  per = per < 256 ? 256 : per;
  per = (per + 127) / 128 * 128;
  const int k_lo = split * per;
  const int k_hi = (k_lo + per) < row.n_keys ? (k_lo + per) : row.n_keys;

  // ---- the R query heads: rotate (tail rows), round to bf16 like the prefill path, one scale per head, two e4m3 terms ----
  for (int idx = tid; idx < R * (HD / 2); idx += 256) {
    const int r = idx / (HD / 2), i = idx % (HD / 2);
    const bf16_t *qp = p.q + (int64_t)row.q_row * q_dim + (kvh * R + r) * HD;
    float x1 = bf16_to_f32(qp[i]), x2 = bf16_to_f32(qp[i + HD / 2]);
    if (row.cs_row >= 0) {
      const float2 c = p.cos_sin[(int64_t)row.cs_row * (HD / 2) + i];
      const float y1 = x1 * c.x - x2 * c.y, y2 = x2 * c.x + x1 * c.y;
      x1 = bf16_to_f32(f32_to_bf16(y1)); x2 = bf16_to_f32(f32_to_bf16(y2));
    }
    q32[r][i] = x1; q32[r][i + HD / 2] = x2;
  }
  __syncthreads();
  for (int r = wave; r < R; r += 4) {
    float a = 0.f;
    for (int d = lane; d < HD; d += 64) a = fmaxf(a, fabsf(q32[r][d]));
    a = wave_max(a);
    if (lane == 0) q_scale[r] = a > 0.f ? a / 448.0f : 1.0f;
  }
  __syncthreads();
  for (int idx = tid; idx < 16 * HD; idx += 256) {
    const int r = idx / HD, d = idx % HD;
    unsigned char hi = 0, lo = 0;
    if (r < R) {
      const float v = q32[r][d] / q_scale[r];
      const int h = __builtin_amdgcn_cvt_pk_fp8_f32(v, 0.f, 0, false);
      const int l = __builtin_amdgcn_cvt_pk_fp8_f32(v - __builtin_amdgcn_cvt_f32_fp8(h, 0), 0.f, 0, false);
      hi = (unsigned char)(h & 0xff); lo = (unsigned char)(l & 0xff);
    }
    q8[0][r][d] = hi; q8[1][r][d] = lo;
  }
  __syncthreads();
  fp8x8_t qh[NM], ql[NM];   // second operand of score instruction m: q[r = l16][d = kq*KB + 8m .. +7]
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    qh[m] = *(const fp8x8_t *)&q8[0][l16][kq * KB + 8 * m];
    ql[m] = *(const fp8x8_t *)&q8[1][l16][kq * KB + 8 * m];
  }
  const float sc = 1.4426950408889634f * rsqrtf((float)HD);
  const float col_scale = l16 < R ? q_scale[l16 < R ? l16 : 0] * sc * (per_slot ? 1.f : p.scale_k[kvh]) : 0.f;
  const float vs_head = per_slot ? 1.f : p.scale_v[kvh];

  const int32_t *bt = p.block_tables + (int64_t)row.seq * p.max_blocks_per_seq;
  const int64_t tok_stride = (int64_t)p.n_kv_heads * HD;   // bytes between tokens of a block
  const uint8_t *ck = (const uint8_t *)p.cache_k + (int64_t)kvh * HD, *cv = (const uint8_t *)p.cache_v + (int64_t)kvh * HD;

  floatx4 o[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) o[db] = floatx4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;   // of column r = l16 (the four lanes of a column agree on m_run)

  // this lane's part of the step that starts at key `base` (a multiple of 32): K bytes of key base + 16 kb + l16,
  // 16-byte pieces of the V tile; keys at or past k_hi read the last visible key's data (masked below)
  uint2 kreg[2][NM];
  u32x4_t vreg[V_IT];   // (a native vector type: as an array of HIP's uint4 structs, written inside the lambda below, it stayed in scratch memory)
  int blk_of[2];          // physical blocks of the two 16-key halves (wave-uniform)
  auto load_step = [&](int base) __attribute__((always_inline)) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      int key0 = base + 16 * kb;
      key0 = key0 < k_hi ? key0 : ((k_hi - 1) & ~15);
      int blk = bt[key0 >> 4];
      blk = ((unsigned)blk < (unsigned)p.n_blocks) ? blk : 0;   // bad ids are flagged by the plan kernel; never dereference them
      blk_of[kb] = blk;
      int key = key0 + l16;
      key = key < k_hi ? key : k_hi - 1;
      const uint8_t *src = ck + ((int64_t)blk * SKV_BLOCK + (key & 15)) * tok_stride + kq * KB;
#pragma unroll
      for (int m = 0; m < NM; ++m) kreg[kb][m] = *(const uint2 *)(src + 8 * m);
    }
#pragma unroll
    for (int i = 0; i < V_IT; ++i) {
      const int c = i * 64 + lane, ch = c % VCH;   // local key c / VCH, 16-byte chunk
      // (a key past the end reads the last visible key, which lies in one of the step's two blocks: no second
      // table lookup, and no branch -- with one, the compiler kept this array in scratch memory and waited
      // for every load before issuing the next)
      const int kl = (c / VCH) < (k_hi - 1 - base) ? (c / VCH) : (k_hi - 1 - base);
      const int blk = (kl >> 4) ? blk_of[1] : blk_of[0];
      vreg[i] = *(const u32x4_t *)(cv + ((int64_t)blk * SKV_BLOCK + ((base + kl) & 15)) * tok_stride + ch * 16);
    }
  };

  unsigned char *vt = v_lds[wave];
  // transposing read of lane group kq: lanes 2j, 2j+1 address the 16 bytes (dims 16 db .. +15) of the key in slot (kq, j)
  const int j_slot = l16 >> 1;
  const int key_slot = j_slot < 4 ? 4 * kq + j_slot : 16 + 4 * kq + (j_slot - 4);
  const unsigned char *vt_lane = vt + key_slot * VS + (lane & 1) * 8;
  typedef int v2i_t __attribute__((ext_vector_type(2)));
  typedef __attribute__((address_space(3))) v2i_t *lds_v2i_ptr;

  if (k_lo + wave * 32 < k_hi) load_step(k_lo + wave * 32);
  for (int base = k_lo + wave * 32; base < k_hi; base += 128) {
    // V tile of this step into the wave's LDS tile (only this wave touches it; a wave's LDS operations run in order)
#pragma unroll
    for (int i = 0; i < V_IT; ++i) {
      const int c = i * 64 + lane;
      *(u32x4_t *)(vt + (c / VCH) * VS + (c % VCH) * 16) = vreg[i];
    }
    fp8x8_t kf[2][NM];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int m = 0; m < NM; ++m) kf[kb][m] = (fp8x8_t)(((unsigned long)kreg[kb][m].y << 32) | kreg[kb][m].x);
    const int blk_cur[2] = {blk_of[0], blk_of[1]};
    load_step(base + 128 < k_hi ? base + 128 : base);   // next step's bytes are in flight during this step's arithmetic (the last step re-reads itself)
    asm volatile("" ::: "memory");

    // scores of keys base + 16 kb + 4 kq + i against head l16
    floatx4 s4[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      s4[kb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        s4[kb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(kf[kb][m], qh[m], s4[kb], 0, 0, 0);
        s4[kb] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(kf[kb][m], ql[m], s4[kb], 0, 0, 0);
      }
    }
    float ksl[8], vsl[8];
    if (per_slot) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int64_t slot0 = (int64_t)blk_cur[kb] * SKV_BLOCK + 4 * kq;
        const float4 a = *(const float4 *)(p.scale_k + slot0), b = *(const float4 *)(p.scale_v + slot0);
        ksl[4 * kb] = a.x; ksl[4 * kb + 1] = a.y; ksl[4 * kb + 2] = a.z; ksl[4 * kb + 3] = a.w;
        vsl[4 * kb] = b.x; vsl[4 * kb + 1] = b.y; vsl[4 * kb + 2] = b.z; vsl[4 * kb + 3] = b.w;
      }
    }
    float sv[8], mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int key = base + 16 * (e >> 2) + 4 * kq + (e & 3);
      float x = s4[e >> 2][e & 3] * col_scale;
      if (per_slot) x *= ksl[e];
      sv[e] = key < k_hi ? x : -INFINITY;
      mx = fmaxf(mx, sv[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    // lazy rescaling: the reference only moves when a score exceeds it by more than 8 (log2 units)
    if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);   // exp2(-inf) = 0 the first time
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) o[db][i] *= alpha;
    }
    // per-slot V scales enter through the weights, relative to the largest scale of the step's keys so that
    // the e4m3 terms keep their precision; the step's product is then added with that scale
    float v_ref = 1.f, v_inv = 1.f;
    if (per_slot) {
      float vm = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) vm = fmaxf(vm, sv[e] == -INFINITY ? 0.f : vsl[e]);
      vm = fmaxf(vm, __shfl_xor(vm, 16));
      vm = fmaxf(vm, __shfl_xor(vm, 32));
      v_ref = vm;
      v_inv = vm > 0.f ? 1.f / vm : 0.f;
    }
    float pw[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float w = (sv[e] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sv[e] - m_run);
      l_run += w;
      pw[e] = per_slot ? w * (vsl[e] * v_inv) : w;
    }
    fp8x8_t ph, pl;
    split_fp8x8(pw, ph, pl);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const v2i_t t = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(vt_lane + db * 16));
      const fp8x8_t vf = make_fp8x8(t.x, t.y);
      if (per_slot) {
        floatx4 acc = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(vf, ph, floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(vf, pl, acc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) o[db][i] += v_ref * acc[i];
      } else {
        o[db] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(vf, ph, o[db], 0, 0, 0);
        o[db] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(vf, pl, o[db], 0, 0, 0);
      }
    }
    asm volatile("" ::: "memory");
  }

  // ---- this wave's (o, m, l) of head l16: o[db][i] = O[d = 16 db + 4 kq + i]; then the four waves, as one split ----
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (l16 < R) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) sm[wave][l16][db * 16 + 4 * kq + i] = o[db][i] * vs_head;
    if (kq == 0) { sm[wave][l16][HD] = m_run; sm[wave][l16][HD + 1] = l_run; }
  }
  __syncthreads();
  for (int i = tid; i < R * HD; i += 256) {
    const int r = i / HD, d = i % HD;
    const float mm = fmaxf(fmaxf(sm[0][r][HD], sm[1][r][HD]), fmaxf(sm[2][r][HD], sm[3][r][HD]));
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

// ------------------------------------------------ decode, bf16 cache, MFMA ----
// The same scheme for a bf16 cache: the vector-unit kernel above spends about 30 vector instructions per key and
// query head (bf16 -> fp32 conversions, the dot products' fma and cross-lane sums); here the dot products are
// matrix instructions (v_mfma_f32_16x16x32_bf16) and the vector unit only does the softmax of the R x 32
// scores of a step, whatever R is.  Used for eight query heads per KV head.  grid (n_rows, n_kv_heads, n_split), 4 waves, 32 keys per
// wave and step.
//  * S^T[key][r]: first operand = K rows straight from the cache (a lane reads 64 contiguous bytes of one key,
//    the four lanes of a key its whole 256-byte row; score instruction m takes the lane's m-th 16 bytes, the
//    query operand is laid out to match), second operand = the R query heads in columns 0..R-1 of 16.
//  * O^T[d][r] += V^T[d][key] P^T[key][r]: the V tile is staged row-major in LDS (row stride hd*2 + 32 bytes)
//    and read with the transposing LDS read for 16-bit data (ds_read_b64_tr_b16: lanes 4r..4r+3 of a 16-lane
//    group address the four 8-byte quarters of row r of a 4 x 16 matrix, lane i receives column i), two reads
//    per fragment.  The 32 keys of a step sit in the contraction slots in the order the score instruction
//    leaves them (slot (g, j): key 4g + j for j < 4, key 16 + 4g + j - 4 otherwise), so the softmax weights go
//    from score registers to operand registers in place.
template <int HD, int R>
__global__ __launch_bounds__(256) void attn_decode_mfma_kernel(AttnDecodeParams p) {
  constexpr int NM = HD / 32;          // score instructions per 16-key block
  constexpr int NDB = HD / 16;         // 16-dim blocks of the output
  constexpr int VS = HD * 2 + 32;      // LDS row stride of the V tile in bytes (rows 8 banks apart)
  constexpr int VCH = HD / 8;          // 16-byte chunks per K / V row
  constexpr int V_IT = 32 * VCH / 64;  // 16-byte loads per lane for a 32-key V tile
  __shared__ __align__(16) unsigned char v_lds[4][32 * VS];
  __shared__ __align__(16) bf16_t qs[16][HD];
  __shared__ float sm[4][R][HD + 2];

  const DecodeRow row = p.rows[blockIdx.x];
  const int kvh = blockIdx.y, split = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, kq = lane >> 4;
  const int q_dim = p.n_q_heads * HD;

  // keys of this split: whole 128-key steps, at least 256 keys per split
  int per = (row.n_keys + p.n_split - 1) / p.n_split;
  per = per < 256 ? 256 : per;
  per = (per + 127) / 128 * 128;
  const int k_lo = split * per;
  const int k_hi = (k_lo + per) < row.n_keys ? (k_lo + per) : row.n_keys;

  // ---- the R query heads as bf16 rows 0..R-1 of a 16-row operand (the rest zero); tail rows are rotated here ----
  for (int idx = tid; idx < 16 * (HD / 2); idx += 256) {
    const int r = idx / (HD / 2), i = idx % (HD / 2);
    bf16_t b1 = 0, b2 = 0;
    if (r < R) {
      const bf16_t *qp = p.q + (int64_t)row.q_row * q_dim + (kvh * R + r) * HD;
      b1 = qp[i]; b2 = qp[i + HD / 2];
      if (row.cs_row >= 0) {
        const float x1 = bf16_to_f32(b1), x2 = bf16_to_f32(b2);
        const float2 c = p.cos_sin[(int64_t)row.cs_row * (HD / 2) + i];
        b1 = f32_to_bf16(x1 * c.x - x2 * c.y); b2 = f32_to_bf16(x2 * c.x + x1 * c.y);   // q is held in bf16 like the prefill path's
      }
    }
    qs[r][i] = b1; qs[r][i + HD / 2] = b2;
  }
  __syncthreads();
  bf16x8 qf[NM];   // second operand of score instruction m: q[r = l16][d = 32 kq + 8 m .. +7]
#pragma unroll
  for (int m = 0; m < NM; ++m) qf[m] = *(const bf16x8 *)&qs[l16][kq * (HD / 4) + 8 * m];
  const float sc = 1.4426950408889634f * rsqrtf((float)HD);

  const int32_t *bt = p.block_tables + (int64_t)row.seq * p.max_blocks_per_seq;
  const int64_t tok_stride = (int64_t)p.n_kv_heads * HD * 2;   // bytes between tokens of a block
  const unsigned char *ck = (const unsigned char *)p.cache_k + (int64_t)kvh * HD * 2, *cv = (const unsigned char *)p.cache_v + (int64_t)kvh * HD * 2;

  floatx4 o[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) o[db] = floatx4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;   // of column r = l16 (the four lanes of a column agree on m_run)

  // this lane's part of the step that starts at key `base` (a multiple of 32): 64 bytes of key base + 16 kb + l16,
  // 16-byte pieces of the V tile; keys at or past k_hi read the last visible key's data (masked below)
  u32x4_t kreg[2][NM];
  u32x4_t vreg[V_IT];   // (a native vector type: as an array of HIP's uint4 structs, written inside the lambda below, it stayed in scratch memory)
  auto load_step = [&](int base) __attribute__((always_inline)) {
    int blk_of[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      int key0 = base + 16 * kb;
      key0 = key0 < k_hi ? key0 : ((k_hi - 1) & ~15);
      int blk = bt[key0 >> 4];
      blk = ((unsigned)blk < (unsigned)p.n_blocks) ? blk : 0;   // bad ids are flagged by the plan kernel; never dereference them
      blk_of[kb] = blk;
      int key = key0 + l16;
      key = key < k_hi ? key : k_hi - 1;
      const unsigned char *src = ck + ((int64_t)blk * SKV_BLOCK + (key & 15)) * tok_stride + kq * (HD / 2);
#pragma unroll
      for (int m = 0; m < NM; ++m) kreg[kb][m] = *(const u32x4_t *)(src + 16 * m);
    }
#pragma unroll
    for (int i = 0; i < V_IT; ++i) {
      const int c = i * 64 + lane, ch = c % VCH;   // local key c / VCH, 16-byte chunk
      // (a key past the end reads the last visible key, which lies in one of the step's two blocks: no second
      // table lookup, and no branch -- with one, the compiler kept this array in scratch memory and waited
      // for every load before issuing the next)
      const int kl = (c / VCH) < (k_hi - 1 - base) ? (c / VCH) : (k_hi - 1 - base);
      const int blk = (kl >> 4) ? blk_of[1] : blk_of[0];
      vreg[i] = *(const u32x4_t *)(cv + ((int64_t)blk * SKV_BLOCK + ((base + kl) & 15)) * tok_stride + ch * 16);
    }
  };

  unsigned char *vt = v_lds[wave];
  // transposing reads of lane group kq: lanes 4r..4r+3 address the 32 bytes (dims 16 db .. +15) of key 4 kq + r
  // (first read) and of key 16 + 4 kq + r (second read)
  const unsigned char *vt_lane = vt + (4 * kq + (l16 >> 2)) * VS + (l16 & 3) * 8;
  typedef short v4s_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) v4s_t *lds_v4s_ptr;

  if (k_lo + wave * 32 < k_hi) load_step(k_lo + wave * 32);
  for (int base = k_lo + wave * 32; base < k_hi; base += 128) {
    // V tile of this step into the wave's LDS tile (only this wave touches it; a wave's LDS operations run in order)
#pragma unroll
    for (int i = 0; i < V_IT; ++i) {
      const int c = i * 64 + lane;
      *(u32x4_t *)(vt + (c / VCH) * VS + (c % VCH) * 16) = vreg[i];
    }
    bf16x8 kf[2][NM];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int m = 0; m < NM; ++m) kf[kb][m] = __builtin_bit_cast(bf16x8, kreg[kb][m]);
    load_step(base + 128 < k_hi ? base + 128 : base);   // next step's bytes are in flight during this step's arithmetic (the last step re-reads itself)
    asm volatile("" ::: "memory");

    // scores of keys base + 16 kb + 4 kq + i against head l16
    floatx4 s4[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      s4[kb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < NM; ++m) s4[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][m], qf[m], s4[kb], 0, 0, 0);
    }
    float sv[8], mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int key = base + 16 * (e >> 2) + 4 * kq + (e & 3);
      sv[e] = key < k_hi ? s4[e >> 2][e & 3] * sc : -INFINITY;
      mx = fmaxf(mx, sv[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    // lazy rescaling: the reference only moves when a score exceeds it by more than 8 (log2 units)
    if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);   // exp2(-inf) = 0 the first time
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) o[db][i] *= alpha;
    }
    bf16x8 pb;   // the weights as second operand: contraction slot (kq, e)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float w = (sv[e] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sv[e] - m_run);
      l_run += w;
      pb[e] = (__bf16)w;
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const v4s_t t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(vt_lane + db * 32));
      const v4s_t t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(vt_lane + 16 * VS + db * 32));
      typedef short v8s_t __attribute__((ext_vector_type(8)));
      const v8s_t t = {t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]};
      o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t), pb, o[db], 0, 0, 0);
    }
    asm volatile("" ::: "memory");
  }

  // ---- this wave's (o, m, l) of head l16: o[db][i] = O[d = 16 db + 4 kq + i]; then the four waves, as one split ----
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (l16 < R) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) sm[wave][l16][db * 16 + 4 * kq + i] = o[db][i];
    if (kq == 0) { sm[wave][l16][HD] = m_run; sm[wave][l16][HD + 1] = l_run; }
  }
  __syncthreads();
  for (int i = tid; i < R * HD; i += 256) {
    const int r = i / HD, d = i % HD;
    const float mm = fmaxf(fmaxf(sm[0][r][HD], sm[1][r][HD]), fmaxf(sm[2][r][HD], sm[3][r][HD]));
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
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) n_cu = 256;
  }
  // two resident workgroups per CU (a multiple of 8, so every XCD's queue has its workgroups)
  dim3 grid((unsigned)(2 * n_cu));
  if (p.head_dim == 128) {
    constexpr int SMEM = 2 * (BKV * 128 * 2 + 128 * BKV * 2);
    static bool set = false;
    if (!set) {
      hipError_t e = hipFuncSetAttribute((const void *)attn_prefill_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
      if (e != hipSuccess) return (int)e;
      set = true;
    }
    hipLaunchKernelGGL(attn_prefill_kernel<128>, grid, dim3(256), SMEM, st, p);
  } else {
    constexpr int SMEM = 2 * (BKV * 64 * 2 + 64 * BKV * 2);
    hipLaunchKernelGGL(attn_prefill_kernel<64>, grid, dim3(256), SMEM, st, p);
  }
  return 0;
}

template <int HD>
static int launch_decode_hd(const AttnDecodeParams &p, hipStream_t st) {
  dim3 grid(p.n_rows, p.n_kv_heads, p.n_split);
  const int R = p.n_q_heads / p.n_kv_heads;
  if (p.fp8) {   // e4m3 cache: the codes go to the matrix unit as they are
    switch (R) {
      case 1: hipLaunchKernelGGL((attn_decode_fp8_kernel<HD, 1>), grid, dim3(256), 0, st, p); break;
      case 2: hipLaunchKernelGGL((attn_decode_fp8_kernel<HD, 2>), grid, dim3(256), 0, st, p); break;
      case 4: hipLaunchKernelGGL((attn_decode_fp8_kernel<HD, 4>), grid, dim3(256), 0, st, p); break;
      case 8: hipLaunchKernelGGL((attn_decode_fp8_kernel<HD, 8>), grid, dim3(256), 0, st, p); break;
      default: return -1;
    }
    return 0;
  }
  // eight query heads per KV head: the matrix-unit form (its cost does not grow with the number of heads; measured on
  // 64 rows x 2048 keys 175 against 254 us per call; with four heads the vector-unit form is 7 % ahead)
  if (R == 8) {
    hipLaunchKernelGGL((attn_decode_mfma_kernel<HD, 8>), grid, dim3(256), 0, st, p);
    return 0;
  }
  switch (R) {
    case 1: hipLaunchKernelGGL((attn_decode_kernel<HD, 1>), grid, dim3(256), 0, st, p); break;
    case 2: hipLaunchKernelGGL((attn_decode_kernel<HD, 2>), grid, dim3(256), 0, st, p); break;
    case 4: hipLaunchKernelGGL((attn_decode_kernel<HD, 4>), grid, dim3(256), 0, st, p); break;
    default: return -1;
  }
  return 0;
}
int launch_attention_decode(const AttnDecodeParams &p, hipStream_t st) {
  if (p.n_rows <= 0) return 0;
  return p.head_dim == 128 ? launch_decode_hd<128>(p, st) : launch_decode_hd<64>(p, st);
}
