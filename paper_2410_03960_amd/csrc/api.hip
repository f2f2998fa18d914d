// C ABI of libswiftkv: context, workspace layout, and the stream-ordered driver
// of the SwiftKV prefill forward pass (layers 1..l on all new tokens, fused KV
// projection of the later layers from the layer-l output, last-token tail).
#include "../../include/swiftkv.h"
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <array>
#include <vector>

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t _e = (expr);                                                               \
    if (_e != hipSuccess) return fail(SWIFTKV_EHIP, "%s: %s", #expr, hipGetErrorString(_e)); \
  } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
constexpr int PIN_SLOTS = 8;

enum TimeClass { TC_QKV = 0, TC_O, TC_GATEUP, TC_DOWN, TC_KV, TC_ATTN, TC_OTHER, TC_TAIL, TC_NORM, TC_COMMIT, TC_COUNT };
static_assert(TC_COUNT == SWIFTKV_N_TIME_CLASSES, "time classes");

struct Layout {  // byte offsets into the workspace
  int64_t T = 0;
  int32_t B = 0;
  int64_t vt_ld = 0;
  int32_t n_qblocks = 0, n_kvtiles = 0, n_dec = 0, n_gtiles = 0;
  int64_t kcat_rows = 0;   // rows of the K buffer gathered from the cache (prompt chunks over a cached prefix), else 0
  size_t err, meta, positions, seq_of, last_rows, slots, cos_sin, h, a, rstd, ssq, q, k, v, o, vt, kcat, z, stage, amax, qkv32, skpart, ee_logits, ee_flags;
  size_t th, ta, tq, to, tz, partial, total;
  // offsets (in int32 units) inside the meta block copied from the host
  size_t m_cu, m_ctx, m_qblocks, m_kvtiles, m_dec, m_tail, m_gtiles, m_words;
};

}  // namespace

struct swiftkv_ctx {
  swiftkv_model_cfg cfg;
  int32_t l, g, P, C;
  int device;
  std::vector<const bf16_t *> norm1, wq, wk, wv, wo, norm2, wgate, wup, wdown;
  const bf16_t *embed, *final_norm, *lm_head;
  // everything below up to kvf_pack points into the caller's pack buffer
  std::vector<const bf16_t *const *> qkv_tab, gu_tab;   // row-block pointer tables (16 rows per entry)
  bf16_t *kv_pack = nullptr;   // [P * 2 * kv_dim, hidden]: leaders' [W_K; W_V] with their norm gain folded in
  // QKV, O, gate/up (interleaved) and down weights of the full layers (< l) in MFMA fragment order, or null
  bool have_wpack = false;
  std::vector<const bf16_t *> qkv_pack, wo_pack, gu_pack, down_pack;
  const bf16_t *kvf_pack = nullptr;   // the fused KV operand (kv_pack) in fragment order
  // pinned staging ring for the per-call plan words: a slot is reused only after the copy that read it has run
  unsigned char *pin = nullptr;
  size_t pin_slot_bytes = 0;
  int pin_next = 0;
  hipEvent_t pin_ev[PIN_SLOTS] = {};
  bool pin_used[PIN_SLOTS] = {};
  // simple early exit of the continuing tokens (off unless swiftkv_set_early_exit was called)
  const bf16_t *ee_gain = nullptr, *ee_head = nullptr;
  float ee_threshold = 0.f;
  Layout last;
  bool have_last = false;
  // timing
  uint32_t timing = 0;   // bit c set: launches of time class c are bracketed by events
  std::vector<hipEvent_t> ev;
  std::vector<int> ev_class;
  size_t ev_used = 0;
  ~swiftkv_ctx() {   // host memory and events only
    if (pin) (void)hipHostFree(pin);
    for (hipEvent_t e : pin_ev)
      if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  }
};

namespace {

constexpr int MAX_SPLIT = 32;
constexpr int SKINNY_MAX_ROWS = 80;   // batches up to this many tokens run every GEMM on the weight-streaming kernel

Layout make_layout(const swiftkv_ctx *c, int64_t T, int32_t B, int64_t vt_ld, int32_t nqb, int32_t nkt,
                   int32_t ndec, bool fp8, int64_t kcat_rows = 0, int32_t ngt = 0) {
  const swiftkv_model_cfg &m = c->cfg;
  const int64_t d = m.hidden, qd = (int64_t)m.n_q_heads * m.head_dim, kvd = (int64_t)m.n_kv_heads * m.head_dim;
  Layout L;
  L.T = T; L.B = B; L.vt_ld = vt_ld; L.n_qblocks = nqb; L.n_kvtiles = nkt; L.n_dec = ndec; L.n_gtiles = ngt; L.kcat_rows = kcat_rows;
  size_t w = 0;
  L.m_cu = w; w += B + 1;
  L.m_ctx = w; w += B;
  w = (w + 3) / 4 * 4;
  L.m_qblocks = w; w += (size_t)nqb * 8;
  L.m_kvtiles = w; w += (size_t)nkt * 4;
  w = (w + 3) / 4 * 4;
  L.m_dec = w; w += (size_t)ndec * 8;
  L.m_tail = w; w += (size_t)B * 8;
  L.m_gtiles = w; w += (size_t)ngt * 8;
  L.m_words = w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  L.err = take(256);
  L.meta = take(L.m_words * 4);
  L.positions = take(T * 4);
  L.seq_of = take(T * 4);
  L.last_rows = take((size_t)B * 4);
  L.slots = take(T * 8);
  L.cos_sin = take(T * (m.head_dim / 2) * 8);
  L.h = take(T * d * 4);      // residual stream, fp32
  L.a = take(T * d * 2);      // bf16 operand of the next projection (normed rows, or rows times the norm gain)
  L.rstd = take(T * 4);
  L.ssq = take((size_t)((d + 63) / 64) * T * 4);   // sums of squares per 64-column block from the residual epilogues
  L.q = take(T * qd * 2);
  L.k = take(T * kvd * 2);
  L.v = take(T * kvd * 2);
  L.o = take(T * qd * 2);
  L.vt = take((size_t)kvd * vt_ld * 2);
  L.kcat = take((size_t)kcat_rows * kvd * 2);
  L.z = take(T * (int64_t)m.ffn * 2);
  L.stage = take(fp8 ? T * (int64_t)c->P * 2 * kvd * 2 : 0);
  L.amax = take(fp8 ? (size_t)c->C * 2 * m.n_kv_heads * 4 : 0);
  L.ee_logits = take(c->ee_head ? (size_t)B * m.vocab * 4 : 0);   // logits of the extra head
  L.ee_flags = take((size_t)B * 4);
  L.skpart = take(SKINNY_PARTIAL_BYTES);   // K-split partial sums of the weight-streaming GEMMs
  L.qkv32 = take((size_t)std::min<int64_t>(T, SKINNY_MAX_ROWS) * (qd + 2 * kvd) * 4);   // fp32 Q, K, V of few-row batches
  L.th = take((size_t)B * d * 4);
  L.ta = take((size_t)B * std::max<int64_t>(d, qd) * 2);
  L.tq = take((size_t)B * qd * 2);
  L.to = take((size_t)B * qd * 2);
  L.tz = take((size_t)B * m.ffn * 2);
  L.partial = take((size_t)std::max(B, ndec) * m.n_q_heads * MAX_SPLIT * (m.head_dim + 2) * 4);
  L.total = off;
  return L;
}

struct Timer {
  swiftkv_ctx *c;
  hipStream_t st;
  void begin(int cls) {
    if (!((c->timing >> cls) & 1u)) return;
    if (c->ev_used + 2 > c->ev.size()) {
      for (int i = 0; i < 64; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        c->ev.push_back(e);
      }
    }
    c->ev_class.push_back(cls);
    (void)hipEventRecord(c->ev[c->ev_used++], st);
  }
  void end() {
    if (!c->timing || (c->ev_used & 1) == 0) return;
    (void)hipEventRecord(c->ev[c->ev_used++], st);
  }
};

int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SWIFTKV_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return 0;
}

// Key splits of the single-query attention: about 1024 workgroups (four per CU, all resident at once:
// measured on 64 rows x 8 KV heads over 2048 keys, 2 splits 118 us, 3 splits 131, 4 splits 125, 1 split
// 141 per launch), no workgroup walking more than about 2048 keys of the longest row (one long row among
// short ones would otherwise finish alone), none fewer than 64.
int pick_split(int rows, int n_kv_heads, int max_keys) {
  const int want = (1024 + rows * n_kv_heads / 2) / (rows * n_kv_heads);
  const int by_len = (max_keys + 1023) / 2048;
  const int cap = std::max(1, max_keys / 64);
  return std::max(1, std::min({std::max(want, by_len), cap, MAX_SPLIT}));
}

struct HostPlan {
  std::vector<int32_t> meta;
  int64_t T = 0, vt_ld = 0, kcat_rows = 0;
  int32_t nqb = 0, nkt = 0, ndec = 0, ngt = 0, max_keys_dec = 0, max_keys_tail = 0;
  bool chunked = false;   // some sequence brings several new tokens on top of a cached context
};

// Host side of the plan: cumulative lengths, 128-query blocks (longest first),
// 64-token KV tiles, the decode rows (one new token on a cached context) and the
// tail rows (last new token of every sequence).  When some sequence brings several
// new tokens on top of a cached context, the prefill attention of every multi-token
// sequence reads K and V^T gathered from the paged cache (64-position gather tiles
// over positions 0 .. context + new - 1) instead of the QKV GEMM's own output.
int build_host_plan(const swiftkv_ctx *c, const int32_t *seq_lens, const int32_t *ctx_lens, int32_t B,
                    int32_t max_blocks_per_seq, HostPlan &hp, Layout &L, bool fp8) {
  std::vector<int64_t> cu(B + 1, 0);
  std::vector<int32_t> vt0(B, -1);
  int64_t vt_cols = 0;
  struct QB { int32_t row0, q0, n, seq_row0, vt_col0, q_last_row; };
  std::vector<QB> qbs;
  std::vector<int32_t> kvt, dec, tail, gt;
  int64_t kcat_rows = 0;
  for (int b = 0; b < B; ++b)
    if (ctx_lens && ctx_lens[b] > 0 && seq_lens[b] > 1) hp.chunked = true;
  for (int b = 0; b < B; ++b) {
    const int64_t n = seq_lens[b], ctx = ctx_lens ? ctx_lens[b] : 0;
    if (n < 1) return fail(SWIFTKV_EINVAL, "seq_lens[%d] = %lld must be >= 1", b, (long long)n);
    if (ctx < 0) return fail(SWIFTKV_EINVAL, "context_lens[%d] is negative", b);
    if ((ctx + n + SKV_BLOCK - 1) / SKV_BLOCK > max_blocks_per_seq)
      return fail(SWIFTKV_ENOSPC, "sequence %d needs %lld blocks, block table has %d", b,
                  (long long)((ctx + n + SKV_BLOCK - 1) / SKV_BLOCK), max_blocks_per_seq);
    cu[b + 1] = cu[b] + n;
    if (cu[b + 1] > 0x7fffffff / 2) return fail(SWIFTKV_EINVAL, "too many tokens");
    const int32_t row0 = (int32_t)cu[b];
    const bool prompt = ctx == 0 || n > 1;
    if (prompt) {
      const int64_t keys = ctx + n;
      vt0[b] = (int32_t)vt_cols;
      vt_cols += ((hp.chunked ? keys : n) + 63) / 64 * 64;
      int32_t k_row0 = row0;
      if (hp.chunked) {
        k_row0 = (int32_t)kcat_rows;
        for (int64_t p0 = 0; p0 < keys; p0 += 64)
          gt.insert(gt.end(), {b, (int32_t)p0, (int32_t)std::min<int64_t>(64, keys - p0), (int32_t)(k_row0 + p0), (int32_t)(vt0[b] + p0), 0, 0, 0});
        kcat_rows += keys;
        if (kcat_rows > 0x7fffffff / 2 || vt_cols > 0x7fffffff / 2) return fail(SWIFTKV_EINVAL, "too many cached + new tokens");
      }
      for (int64_t q0 = 0; q0 < n; q0 += 128)
        qbs.push_back({(int32_t)(row0 + q0), (int32_t)(ctx + q0), (int32_t)keys, k_row0, vt0[b], (int32_t)(row0 + n - 1)});
    } else {
      dec.insert(dec.end(), {row0, row0, b, (int32_t)(ctx + 1), -1, 0, 0, 0});
      hp.max_keys_dec = std::max<int32_t>(hp.max_keys_dec, (int32_t)(ctx + 1));
    }
    for (int64_t p0 = 0; p0 < n; p0 += 64)
      kvt.insert(kvt.end(), {(int32_t)(row0 + p0), (int32_t)std::min<int64_t>(64, n - p0), (prompt && !hp.chunked) ? (int32_t)(vt0[b] + p0) : -1, 0});
    // tail row: q row b of the tail buffer, rotated with the last token's angles
    tail.insert(tail.end(), {b, b, b, (int32_t)(ctx + n), (int32_t)(cu[b + 1] - 1), 0, 0, 0});
    hp.max_keys_tail = std::max<int32_t>(hp.max_keys_tail, (int32_t)(ctx + n));
  }
  std::stable_sort(qbs.begin(), qbs.end(), [](const QB &a, const QB &b) {
    return std::min(a.q0 + 128, a.n) > std::min(b.q0 + 128, b.n);
  });
  hp.T = cu[B];
  hp.vt_ld = std::max<int64_t>(vt_cols, 64);
  hp.nqb = (int32_t)qbs.size();
  hp.nkt = (int32_t)(kvt.size() / 4);
  hp.ndec = (int32_t)(dec.size() / 8);
  hp.ngt = (int32_t)(gt.size() / 8);
  hp.kcat_rows = kcat_rows;
  L = make_layout(c, hp.T, B, hp.vt_ld, hp.nqb, hp.nkt, hp.ndec, fp8, kcat_rows, hp.ngt);
  hp.meta.assign(L.m_words, 0);
  for (int b = 0; b <= B; ++b) hp.meta[L.m_cu + b] = (int32_t)cu[b];
  for (int b = 0; b < B; ++b) hp.meta[L.m_ctx + b] = ctx_lens ? ctx_lens[b] : 0;
  for (size_t i = 0; i < qbs.size(); ++i) {
    int32_t *q = &hp.meta[L.m_qblocks + i * 8];
    q[0] = qbs[i].row0; q[1] = qbs[i].q0; q[2] = qbs[i].n; q[3] = qbs[i].seq_row0; q[4] = qbs[i].vt_col0; q[5] = qbs[i].q_last_row;
  }
  std::copy(kvt.begin(), kvt.end(), hp.meta.begin() + L.m_kvtiles);
  std::copy(dec.begin(), dec.end(), hp.meta.begin() + L.m_dec);
  std::copy(tail.begin(), tail.end(), hp.meta.begin() + L.m_tail);
  std::copy(gt.begin(), gt.end(), hp.meta.begin() + L.m_gtiles);
  return 0;
}

int validate_cache(const swiftkv_ctx *c, const swiftkv_kv_cache *kv) {
  if (!kv || !kv->data || !kv->block_tables) return fail(SWIFTKV_EINVAL, "kv cache descriptor has null pointers");
  if (kv->block_size != SKV_BLOCK) return fail(SWIFTKV_EINVAL, "block_size must be 16, got %d", kv->block_size);
  if (kv->n_cache_layers != c->C)
    return fail(SWIFTKV_EINVAL, "cache has %d layers, l=%d g=%d needs %d", kv->n_cache_layers, c->l, c->g, c->C);
  if (kv->n_blocks < 1 || kv->max_blocks_per_seq < 1) return fail(SWIFTKV_EINVAL, "empty block pool or table");
  if (kv->dtype != SWIFTKV_KV_BF16 && kv->dtype != SWIFTKV_KV_FP8_E4M3) return fail(SWIFTKV_EINVAL, "bad kv dtype");
  if (kv->dtype == SWIFTKV_KV_FP8_E4M3 && !kv->scales) return fail(SWIFTKV_EINVAL, "FP8 cache needs scales");
  if (kv->dtype == SWIFTKV_KV_FP8_E4M3 && kv->scale_mode != SWIFTKV_SCALE_COMPUTE_ABSMAX && kv->scale_mode != SWIFTKV_SCALE_USE_GIVEN &&
      kv->scale_mode != SWIFTKV_SCALE_PER_TOKEN)
    return fail(SWIFTKV_EINVAL, "bad scale_mode");
  return 0;
}

// everything from the plan up to the cache of layers > l; shared by the two entry points
struct Run {
  swiftkv_ctx *c;
  const swiftkv_kv_cache *kv;
  unsigned char *ws;
  Layout L;
  HostPlan hp;
  hipStream_t st;
  bool fp8;
  bool per_token;             // FP8 with one scale per cache slot
  int64_t n_slots;
  size_t esz;                 // cache element bytes
  int64_t plane, layer_stride;  // elements per K (or V) plane / per cache layer

  template <class T> T *at(size_t off) const { return (T *)(ws + off); }
  const int32_t *meta(size_t word) const { return at<int32_t>(L.meta) + word; }
  // scales of cache layer c: [2][Hkv], or [2][n_slots] with per-token scales
  float *layer_scales(int c_layer) const {
    return kv->scales + (int64_t)c_layer * 2 * (per_token ? n_slots : (int64_t)c->cfg.n_kv_heads);
  }
  int fp8_kind() const { return !fp8 ? 0 : (per_token ? 2 : 1); }
  void *cache_plane(int c_layer, int kvsel) const {
    return (unsigned char *)kv->data + ((int64_t)c_layer * layer_stride + (int64_t)kvsel * plane) * esz;
  }
};

// (Re)allocate the pinned staging ring with slots of at least `need` bytes.  Host memory only.
int pin_reserve(swiftkv_ctx *c, size_t need) {
  if (c->pin && need <= c->pin_slot_bytes) return 0;
  for (int i = 0; i < PIN_SLOTS; ++i)
    if (c->pin_used[i]) { HIP_TRY(hipEventSynchronize(c->pin_ev[i])); c->pin_used[i] = false; }
  if (c->pin) { HIP_TRY(hipHostFree(c->pin)); c->pin = nullptr; c->pin_slot_bytes = 0; }
  const size_t slot = align_up(std::max<size_t>(2 * need, 64 << 10), 4096);
  HIP_TRY(hipHostMalloc((void **)&c->pin, slot * PIN_SLOTS, hipHostMallocDefault));
  c->pin_slot_bytes = slot;
  for (int i = 0; i < PIN_SLOTS; ++i)
    if (!c->pin_ev[i]) HIP_TRY(hipEventCreateWithFlags(&c->pin_ev[i], hipEventDisableTiming));
  return 0;
}

int run_plan(Run &r, const int32_t *token_ids) {
  swiftkv_ctx *c = r.c;
  // plan words: host vector -> pinned slot -> device, without waiting for the stream (a slot is only
  // waited for when the ring wraps around onto a copy that has not run yet)
  const size_t bytes = r.hp.meta.size() * 4;
  if (int e = pin_reserve(c, bytes)) return e;
  const int slot = c->pin_next;
  c->pin_next = (slot + 1) % PIN_SLOTS;
  if (c->pin_used[slot]) HIP_TRY(hipEventSynchronize(c->pin_ev[slot]));
  unsigned char *stage = c->pin + (size_t)slot * c->pin_slot_bytes;
  memcpy(stage, r.hp.meta.data(), bytes);
  HIP_TRY(hipMemcpyAsync(r.ws + r.L.meta, stage, bytes, hipMemcpyHostToDevice, r.st));
  HIP_TRY(hipEventRecord(c->pin_ev[slot], r.st));
  c->pin_used[slot] = true;
  launch_fill_u32(r.at<uint32_t>(r.L.err), 0, 16, r.st);   // error flags, and (words 4..12) the attention kernel's item counters
  if (r.fp8) launch_fill_u32(r.at<uint32_t>(r.L.amax), 0, (int64_t)c->C * 2 * c->cfg.n_kv_heads, r.st);
  PlanParams pp{};
  pp.T = (int32_t)r.L.T; pp.B = r.L.B; pp.head_dim = c->cfg.head_dim; pp.n_blocks = r.kv->n_blocks;
  pp.max_blocks_per_seq = r.kv->max_blocks_per_seq; pp.vocab = c->cfg.vocab; pp.rope_theta = c->cfg.rope_theta;
  pp.cu_seqlens = r.meta(r.L.m_cu); pp.context_lens = r.meta(r.L.m_ctx); pp.block_tables = r.kv->block_tables;
  pp.token_ids = token_ids;
  pp.positions = r.at<int32_t>(r.L.positions); pp.seq_of = r.at<int32_t>(r.L.seq_of);
  pp.last_rows = r.at<int32_t>(r.L.last_rows); pp.err_flag = r.at<int32_t>(r.L.err);
  pp.slots = r.at<int64_t>(r.L.slots); pp.cos_sin = r.at<float2>(r.L.cos_sin);
  launch_plan(pp, r.st);
  return check_launch("plan");
}

// Eq. 2 + AcrossKV: one GEMM over the concatenated leader [W_K;W_V] matrices.
// `hidden` = the layer-l output rounded to bf16; 1/rms of its rows is already in the workspace when rstd_ready
int run_fused_kv(Run &r, const bf16_t *hidden, bool rstd_ready, Timer &tm) {
  swiftkv_ctx *c = r.c;
  const swiftkv_model_cfg &m = c->cfg;
  const int kvd = m.n_kv_heads * m.head_dim;
  if (!rstd_ready) {
    tm.begin(TC_NORM);
    launch_rstd(hidden, r.at<float>(r.L.rstd), (int32_t)r.L.T, m.hidden, m.rms_eps, r.st);
    tm.end();
  }
  GemmParams g{};
  g.A = hidden; g.lda = m.hidden; g.M = (int32_t)r.L.T; g.N = c->P * 2 * kvd; g.K = m.hidden;
  g.W = c->kv_pack; g.ldw = m.hidden; g.wpack = c->kvf_pack;   // gains are folded into kv_pack; rstd is applied in the epilogue
  g.rstd = r.at<float>(r.L.rstd); g.cos_sin = r.at<float2>(r.L.cos_sin);
  g.head_dim = m.head_dim; g.q_dim = m.n_q_heads * m.head_dim; g.kv_dim = kvd;
  g.slots = r.at<int64_t>(r.L.slots); g.cache = (bf16_t *)r.kv->data;
  g.cache_layer_stride = r.layer_stride; g.cache_kv_stride = r.plane; g.first_cache_layer = c->l;
  if (r.fp8) {
    g.stage = r.at<bf16_t>(r.L.stage);
    g.amax = r.kv->scale_mode == SWIFTKV_SCALE_COMPUTE_ABSMAX ? r.at<uint32_t>(r.L.amax) : nullptr;
  }
  tm.begin(TC_KV);
  if (launch_gemm(g, EPI_KV, 0, r.st) != 0) return fail(SWIFTKV_EHIP, "fused KV GEMM launch failed");
  tm.end();
  if (int e = check_launch("fused KV GEMM")) return e;
  if (r.fp8) {
    tm.begin(TC_COMMIT);
    for (int p = 0; p < c->P; ++p) {
      const int cl = c->l + p;
      CommitParams cp{};
      cp.tiles = (const KVTile *)r.meta(r.L.m_kvtiles); cp.n_tiles = r.L.n_kvtiles;
      cp.n_kv_heads = m.n_kv_heads; cp.head_dim = m.head_dim;
      cp.k_src = r.at<bf16_t>(r.L.stage) + (int64_t)p * 2 * kvd; cp.v_src = cp.k_src + kvd; cp.ld_src = g.N;
      cp.cache_k = r.cache_plane(cl, 0); cp.cache_v = r.cache_plane(cl, 1);
      cp.slots = r.at<int64_t>(r.L.slots); cp.fp8 = 1;
      cp.compute_scale = r.kv->scale_mode == SWIFTKV_SCALE_COMPUTE_ABSMAX;
      cp.amax = r.at<uint32_t>(r.L.amax) + (int64_t)cl * 2 * m.n_kv_heads;
      cp.scales = r.layer_scales(cl);
      cp.per_token = r.per_token; cp.n_slots = r.n_slots;
      cp.vt = nullptr; cp.writeback = 0;
      if (r.per_token) {
        TokenScaleParams tp{cp.k_src, cp.v_src, cp.ld_src, (int32_t)r.L.T, kvd, cp.slots, cp.scales, r.n_slots};
        launch_token_scales(tp, r.st);
      }
      launch_kv_commit(cp, r.st);
    }
    tm.end();
    if (int e = check_launch("fp8 KV commit")) return e;
  }
  return 0;
}

// n_splits_out (host, may be null): see SkinnyParams -- the consumer of C adds the K splits
int tail_gemm(const swiftkv_ctx *c, const bf16_t *A, int M, int N, int K, const bf16_t *W, const bf16_t *W2,
              const bf16_t *const *gu_tab, void *C, int epi, float *partial, hipStream_t st, int32_t *n_splits_out = nullptr) {
  if (n_splits_out) *n_splits_out = 1;
  if (M <= 80) {
    SkinnyParams s{A, M, N, K, W, W2, C, partial, SKINNY_PARTIAL_BYTES, nullptr, n_splits_out};
    return launch_skinny(s, epi, st);
  }
  GemmParams g{};
  g.A = A; g.lda = K; g.M = M; g.K = K; g.ldw = K; g.C = C;
  if (epi == EPI_SWIGLU) { g.wtab = gu_tab; g.N = 2 * N; g.ldc = N; }
  else { g.W = W; g.N = N; g.ldc = N; }
  (void)c;
  return launch_gemm(g, epi, 2, st);
}

}  // namespace

extern "C" {

const char *swiftkv_last_error(void) { return g_err; }
const char *swiftkv_version(void) { return "swiftkv-gfx950 0.1"; }

// Validation of (shape, l, g) shared by the size calls and swiftkv_create; 0 = fine.
static int check_model(const swiftkv_model_cfg &m, int32_t l, int32_t g) {
  if (m.n_layers < 1 || m.hidden < 16 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.ffn < 16 || m.vocab < 16)
    return fail(SWIFTKV_EINVAL, "bad model shape");
  if (m.head_dim != 64 && m.head_dim != 128) return fail(SWIFTKV_EINVAL, "head_dim must be 64 or 128, got %d", m.head_dim);
  if (m.n_q_heads % m.n_kv_heads) return fail(SWIFTKV_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
  const int R = m.n_q_heads / m.n_kv_heads;
  if (R != 1 && R != 2 && R != 4 && R != 8) return fail(SWIFTKV_EINVAL, "query heads per KV head must be 1, 2, 4 or 8");
  const int qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim;
  if (qd % 128 || kvd % 128) return fail(SWIFTKV_EINVAL, "n_heads*head_dim must be multiples of 128");
  if (m.hidden % 16 || m.ffn % 16 || m.vocab % 16) return fail(SWIFTKV_EINVAL, "hidden, ffn and vocab must be multiples of 16");
  if (l < 1 || l > m.n_layers) return fail(SWIFTKV_EINVAL, "l = %d outside [1, %d]", l, m.n_layers);
  if (g < 1 || (m.n_layers - l) % g) return fail(SWIFTKV_EINVAL, "(n_layers - l) = %d is not divisible by acrosskv_group = %d", m.n_layers - l, g);
  return 0;
}

// Layout of the caller's pack buffer (byte offsets, 256-byte aligned pieces).
struct PackLayout {
  size_t tab_entries, tables, kv_pack, w_pack, min_total, full_total;
  size_t e_qkv, e_o, e_gu, e_dn, per_layer, e_kvf;   // elements of the fragment-order copies
  bool can_pack;
};
static PackLayout pack_layout(const swiftkv_model_cfg &m, int32_t l, int32_t g) {
  PackLayout p{};
  const size_t d = m.hidden, qd = (size_t)m.n_q_heads * m.head_dim, kvd = (size_t)m.n_kv_heads * m.head_dim;
  const size_t P = (size_t)(m.n_layers - l) / g;
  p.tab_entries = (size_t)m.n_layers * ((qd + 2 * kvd) / 16 + 2 * ((size_t)m.ffn / 16)) + 1;
  p.tables = 0;
  p.kv_pack = align_up(p.tab_entries * sizeof(void *));
  p.w_pack = p.kv_pack + align_up(P * 2 * kvd * d * 2);
  p.min_total = p.w_pack;
  p.can_pack = (d % 256) == 0 && (qd % 256) == 0 && (m.ffn % 256) == 0 && (kvd % 128) == 0;
  p.e_qkv = (qd + 2 * kvd) * d; p.e_o = d * qd; p.e_gu = (size_t)2 * m.ffn * d; p.e_dn = d * (size_t)m.ffn;
  p.per_layer = p.e_qkv + p.e_o + p.e_gu + p.e_dn;
  p.e_kvf = P * 2 * kvd * d;
  p.full_total = p.can_pack ? p.w_pack + align_up((p.per_layer * l + p.e_kvf) * 2) : p.min_total;
  return p;
}

size_t swiftkv_pack_bytes(const swiftkv_model_cfg *cfg, int32_t l, int32_t g) {
  if (!cfg || check_model(*cfg, l, g)) return 0;
  return pack_layout(*cfg, l, g).full_total;
}
size_t swiftkv_pack_bytes_min(const swiftkv_model_cfg *cfg, int32_t l, int32_t g) {
  if (!cfg || check_model(*cfg, l, g)) return 0;
  return pack_layout(*cfg, l, g).min_total;
}

int swiftkv_create(swiftkv_ctx **out, const swiftkv_model_cfg *cfg, const swiftkv_weights *w, int32_t l, int32_t g,
                   void *pack_buf, size_t pack_bytes, void *stream) {
  if (!out || !cfg || !w) return fail(SWIFTKV_EINVAL, "null argument");
  *out = nullptr;
  const swiftkv_model_cfg &m = *cfg;
  if (int e = check_model(m, l, g)) return e;
  const int qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim;
  if (!w->embed || !w->final_norm || !w->lm_head || !w->norm1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->norm2 ||
      !w->wgate || !w->wup || !w->wdown)
    return fail(SWIFTKV_EINVAL, "null weight array");
  const PackLayout pl = pack_layout(m, l, g);
  if (!pack_buf || pack_bytes < pl.min_total)
    return fail(SWIFTKV_ENOSPC, "pack buffer has %zu bytes, at least %zu needed (%zu for the fragment-order copies as well)",
                pack_buf ? pack_bytes : (size_t)0, pl.min_total, pl.full_total);
  if (((uintptr_t)pack_buf & 255) != 0) return fail(SWIFTKV_EINVAL, "pack_buf must be 256-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  unsigned char *pb = (unsigned char *)pack_buf;
  std::unique_ptr<swiftkv_ctx> c(new swiftkv_ctx());
  c->cfg = m; c->l = l; c->g = g; c->P = (m.n_layers - l) / g; c->C = l + c->P;
  c->embed = (const bf16_t *)w->embed; c->final_norm = (const bf16_t *)w->final_norm; c->lm_head = (const bf16_t *)w->lm_head;
  auto grab = [&](std::vector<const bf16_t *> &v, const void *const *src) {
    v.resize(m.n_layers);
    for (int j = 0; j < m.n_layers; ++j) v[j] = (const bf16_t *)src[j];
  };
  grab(c->norm1, w->norm1); grab(c->wq, w->wq); grab(c->wk, w->wk); grab(c->wv, w->wv); grab(c->wo, w->wo);
  grab(c->norm2, w->norm2); grab(c->wgate, w->wgate); grab(c->wup, w->wup); grab(c->wdown, w->wdown);
  for (int j = 0; j < m.n_layers; ++j) {
    const bool need_kv = j < l || ((j - l) % g == 0);
    if (!c->norm1[j] || !c->wq[j] || !c->wo[j] || !c->norm2[j] || !c->wgate[j] || !c->wup[j] || !c->wdown[j] ||
        (need_kv && (!c->wk[j] || !c->wv[j])))
      return fail(SWIFTKV_EINVAL, "layer %d has a null weight pointer", j);
  }
  if (hipGetDevice(&c->device) != hipSuccess) return fail(SWIFTKV_EHIP, "no current device");
  if (int e = pin_reserve(c.get(), 0)) return e;
  // ---- row-block pointer tables (16 rows per entry): [W_Q;W_K;W_V] and the 16-row interleave of W_gate/W_up ----
  std::vector<const bf16_t *> tab;
  std::vector<size_t> off_qkv(m.n_layers), off_gu(m.n_layers);
  const int64_t d = m.hidden;
  for (int j = 0; j < m.n_layers; ++j) {
    off_qkv[j] = tab.size();
    for (int r = 0; r < qd; r += 16) tab.push_back(c->wq[j] + (int64_t)r * d);
    for (int r = 0; r < kvd; r += 16) tab.push_back(c->wk[j] ? c->wk[j] + (int64_t)r * d : nullptr);
    for (int r = 0; r < kvd; r += 16) tab.push_back(c->wv[j] ? c->wv[j] + (int64_t)r * d : nullptr);
    off_gu[j] = tab.size();
    for (int r = 0; r < m.ffn; r += 16) {
      tab.push_back(c->wgate[j] + (int64_t)r * d);
      tab.push_back(c->wup[j] + (int64_t)r * d);
    }
  }
  tab.push_back(nullptr);
  if (tab.size() != pl.tab_entries) return fail(SWIFTKV_EINVAL, "internal: table size");
  HIP_TRY(hipMemcpyAsync(pb + pl.tables, tab.data(), tab.size() * sizeof(void *), hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));   // `tab` is pageable host memory: the copy must have read it before it goes away
  const bf16_t *const *base = (const bf16_t *const *)(pb + pl.tables);
  c->qkv_tab.resize(m.n_layers); c->gu_tab.resize(m.n_layers);
  for (int j = 0; j < m.n_layers; ++j) { c->qkv_tab[j] = base + off_qkv[j]; c->gu_tab[j] = base + off_gu[j]; }
  if (c->P > 0) {
    // one operand for the single KV GEMM of Eq. 2: [W_K^j; W_V^j] diag(g1_j) of every group leader j
    c->kv_pack = (bf16_t *)(pb + pl.kv_pack);
    for (int p = 0; p < c->P; ++p) {
      const int j = l + p * g;
      bf16_t *dst = c->kv_pack + (size_t)p * 2 * kvd * d;
      launch_fold_gain(c->wk[j], c->norm1[j], dst, kvd, m.hidden, st);
      launch_fold_gain(c->wv[j], c->norm1[j], dst + (size_t)kvd * d, kvd, m.hidden, st);
    }
  }
  // Fragment-order copies of the large GEMM weights of the layers every token runs, when the caller gave room
  c->qkv_pack.assign(m.n_layers, nullptr); c->wo_pack.assign(m.n_layers, nullptr);
  c->gu_pack.assign(m.n_layers, nullptr); c->down_pack.assign(m.n_layers, nullptr);
  if (pl.can_pack && pack_bytes >= pl.full_total) {
    bf16_t *wp = (bf16_t *)(pb + pl.w_pack);
    const int rope_hd = m.head_dim == 128 ? 128 : 0;   // rotary partner blocks side by side (see pack_w_kernel)
    for (int j = 0; j < l; ++j) {
      bf16_t *pq = wp + (size_t)j * pl.per_layer, *po = pq + pl.e_qkv, *pgu = po + pl.e_o, *pdn = pgu + pl.e_gu;
      launch_pack_w(c->qkv_tab[j], nullptr, d, qd + 2 * kvd, (int32_t)d, rope_hd, pq, st);
      launch_pack_w(nullptr, c->wo[j], qd, (int32_t)d, qd, 0, po, st);
      launch_pack_w(c->gu_tab[j], nullptr, d, 2 * m.ffn, (int32_t)d, 0, pgu, st);
      launch_pack_w(nullptr, c->wdown[j], m.ffn, (int32_t)d, m.ffn, 0, pdn, st);
      c->qkv_pack[j] = pq; c->wo_pack[j] = po; c->gu_pack[j] = pgu; c->down_pack[j] = pdn;
    }
    if (c->P > 0) {
      bf16_t *pk = wp + pl.per_layer * l;
      launch_pack_w(nullptr, c->kv_pack, d, c->P * 2 * kvd, (int32_t)d, rope_hd, pk, st);
      c->kvf_pack = pk;
    }
    c->have_wpack = true;
  }
  if (int e = check_launch("weight packing")) return e;
  HIP_TRY(hipStreamSynchronize(st));
  *out = c.release();
  return SWIFTKV_OK;
}

void swiftkv_destroy(swiftkv_ctx *c) { delete c; }

size_t swiftkv_workspace_bytes_prefix(const swiftkv_ctx *c, int64_t max_tokens, int32_t max_seqs, int32_t kv_dtype,
                                      int64_t max_prefix_tokens) {
  if (!c || max_tokens < 1 || max_seqs < 1 || max_prefix_tokens < 0) return 0;
  const int64_t kcat_rows = max_prefix_tokens > 0 ? max_tokens + max_prefix_tokens : 0;
  const int64_t vt_ld = max_tokens + max_prefix_tokens + 64LL * max_seqs;
  const int32_t nqb = (int32_t)(max_tokens / 128 + max_seqs), nkt = (int32_t)(max_tokens / 64 + max_seqs);
  const int32_t ngt = kcat_rows ? (int32_t)(kcat_rows / 64 + max_seqs) : 0;
  Layout L = make_layout(c, max_tokens, max_seqs, vt_ld, nqb, nkt, max_seqs, kv_dtype == SWIFTKV_KV_FP8_E4M3, kcat_rows, ngt);
  return L.total + 4096;
}

size_t swiftkv_workspace_bytes(const swiftkv_ctx *c, int64_t max_tokens, int32_t max_seqs, int32_t kv_dtype) {
  return swiftkv_workspace_bytes_prefix(c, max_tokens, max_seqs, kv_dtype, 0);
}

int swiftkv_set_early_exit(swiftkv_ctx *c, const void *gain, const void *head, float threshold) {
  if (!c) return fail(SWIFTKV_EINVAL, "null ctx");
  if ((gain == nullptr) != (head == nullptr)) return fail(SWIFTKV_EINVAL, "gain and head must both be given or both be null");
  c->ee_gain = (const bf16_t *)gain; c->ee_head = (const bf16_t *)head; c->ee_threshold = threshold;
  return SWIFTKV_OK;
}

int swiftkv_export_exit_flags(swiftkv_ctx *c, const void *workspace, int32_t *flags_out, void *stream) {
  if (!c || !workspace || !flags_out) return fail(SWIFTKV_EINVAL, "null argument");
  if (!c->have_last) return fail(SWIFTKV_EINVAL, "no prefill has run on this ctx");
  HIP_TRY(hipMemcpyAsync(flags_out, (const unsigned char *)workspace + c->last.ee_flags, (size_t)c->last.B * 4, hipMemcpyDeviceToDevice,
                         (hipStream_t)stream));
  return SWIFTKV_OK;
}

int swiftkv_set_timing(swiftkv_ctx *c, int32_t class_mask) {
  if (!c) return fail(SWIFTKV_EINVAL, "null ctx");
  if (class_mask < 0 || class_mask > SWIFTKV_TIME_ALL) return fail(SWIFTKV_EINVAL, "class_mask %d names no time class", class_mask);
  c->timing = (uint32_t)class_mask;
  c->ev_used = 0;          // (re)start accumulating
  c->ev_class.clear();
  return SWIFTKV_OK;
}

int swiftkv_get_timing(swiftkv_ctx *c, double ms_out[8], int32_t launches_out[8]) {
  if (!c || !ms_out || !launches_out) return fail(SWIFTKV_EINVAL, "null argument");
  for (int i = 0; i < TC_COUNT; ++i) { ms_out[i] = 0; launches_out[i] = 0; }
  if (c->ev_used == 0) return SWIFTKV_OK;
  HIP_TRY(hipEventSynchronize(c->ev[c->ev_used - 1]));
  for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]));
    ms_out[c->ev_class[i / 2]] += ms;
    launches_out[c->ev_class[i / 2]] += 1;
  }
  return SWIFTKV_OK;
}

int swiftkv_flops(const swiftkv_ctx *c, const int32_t *seq_lens, const int32_t *ctx_lens, int32_t B, double *gemm, double *attn) {
  if (!c || !seq_lens || !gemm || !attn) return fail(SWIFTKV_EINVAL, "null argument");
  const swiftkv_model_cfg &m = c->cfg;
  const double d = m.hidden, qd = (double)m.n_q_heads * m.head_dim, kvd = (double)m.n_kv_heads * m.head_dim;
  const double layer = 2 * d * (qd + 2 * kvd) + 2 * d * qd + 6 * d * m.ffn;
  double T = 0, a = 0;
  for (int b = 0; b < B; ++b) {
    const double n = seq_lens[b], ctx = ctx_lens ? ctx_lens[b] : 0;
    T += n;
    a += c->l * 4 * qd * (n * ctx + n * (n + 1) / 2);
    a += (m.n_layers - c->l) * 4 * qd * (ctx + n);
  }
  *gemm = T * (c->l * layer + c->P * 2 * d * 2 * kvd) + B * ((m.n_layers - c->l) * (4 * d * qd + 6 * d * m.ffn) + 2 * d * m.vocab);
  *attn = a;
  return SWIFTKV_OK;
}

static int setup_run(Run &r, swiftkv_ctx *c, const int32_t *seq_lens, int32_t B, const swiftkv_kv_cache *kv,
                     void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !seq_lens || !workspace) return fail(SWIFTKV_EINVAL, "null argument");
  if (B < 1) return fail(SWIFTKV_EINVAL, "n_seqs must be >= 1");
  if (int e = validate_cache(c, kv)) return e;
  r.c = c; r.kv = kv; r.ws = (unsigned char *)workspace; r.st = (hipStream_t)stream;
  r.fp8 = kv->dtype == SWIFTKV_KV_FP8_E4M3;
  r.per_token = r.fp8 && kv->scale_mode == SWIFTKV_SCALE_PER_TOKEN;
  r.n_slots = (int64_t)kv->n_blocks * SKV_BLOCK;
  r.esz = r.fp8 ? 1 : 2;
  r.plane = (int64_t)kv->n_blocks * SKV_BLOCK * c->cfg.n_kv_heads * c->cfg.head_dim;
  r.layer_stride = 2 * r.plane;
  if (r.fp8 && kv->scale_mode == SWIFTKV_SCALE_COMPUTE_ABSMAX && kv->context_lens)
    for (int b = 0; b < B; ++b)
      if (kv->context_lens[b] > 0)
        return fail(SWIFTKV_EINVAL, "FP8 cache with computed per-head scales: sequence %d has %d cached tokens, whose codes were "
                    "stored under other scales (use SWIFTKV_SCALE_USE_GIVEN or SWIFTKV_SCALE_PER_TOKEN)", b, kv->context_lens[b]);
  if (int e = build_host_plan(c, seq_lens, kv->context_lens, B, kv->max_blocks_per_seq, r.hp, r.L, r.fp8)) return e;
  if (r.L.total > workspace_bytes)
    return fail(SWIFTKV_ENOSPC, "workspace has %zu bytes, %zu needed", workspace_bytes, r.L.total);
  if (((uintptr_t)workspace & 255) != 0) return fail(SWIFTKV_EINVAL, "workspace must be 256-byte aligned");
  return 0;
}

int swiftkv_kv_from_hidden(swiftkv_ctx *c, const void *hidden_l, const int32_t *seq_lens, int32_t B,
                           const swiftkv_kv_cache *kv, void *workspace, size_t workspace_bytes, void *stream) {
  Run r;
  if (int e = setup_run(r, c, seq_lens, B, kv, workspace, workspace_bytes, stream)) return e;
  if (!hidden_l) return fail(SWIFTKV_EINVAL, "null hidden_l");
  if (c->P == 0) return fail(SWIFTKV_EINVAL, "l == n_layers: there are no later layers to project for");
  if (int e = run_plan(r, nullptr)) return e;
  Timer tm{c, r.st};
  if (int e = run_fused_kv(r, (const bf16_t *)hidden_l, false, tm)) return e;
  c->last = r.L; c->have_last = true;
  return SWIFTKV_OK;
}

int swiftkv_prefill(swiftkv_ctx *c, const int32_t *token_ids, const int32_t *seq_lens, int32_t B,
                    const swiftkv_kv_cache *kv, float *logits_out, void *workspace, size_t workspace_bytes, void *stream) {
  Run r;
  if (int e = setup_run(r, c, seq_lens, B, kv, workspace, workspace_bytes, stream)) return e;
  if (!token_ids || !logits_out) return fail(SWIFTKV_EINVAL, "null token_ids or logits_out");
  if (c->ee_head && B > 65535) return fail(SWIFTKV_EINVAL, "early exit handles at most 65535 sequences per call");
  const swiftkv_model_cfg &m = c->cfg;
  const int T = (int)r.L.T, d = m.hidden, qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim;
  hipStream_t st = r.st;
  Timer tm{c, st};
  tm.begin(TC_OTHER);
  if (int e = run_plan(r, token_ids)) return e;
  float *h = r.at<float>(r.L.h);             // residual stream, fp32 [T, d]
  launch_embed(token_ids, c->embed, h, T, d, m.vocab, st);
  tm.end();
  bf16_t *ab = r.at<bf16_t>(r.L.a);          // bf16 operand of the projection behind an RMSNorm
  bf16_t *qb = r.at<bf16_t>(r.L.q), *kb = r.at<bf16_t>(r.L.k), *vb = r.at<bf16_t>(r.L.v), *ob = r.at<bf16_t>(r.L.o);
  bf16_t *vt = r.at<bf16_t>(r.L.vt), *zb = r.at<bf16_t>(r.L.z);
  const bool compute_scale = r.fp8 && kv->scale_mode == SWIFTKV_SCALE_COMPUTE_ABSMAX;
  const bool few_rows = T <= SKINNY_MAX_ROWS;
  float *skp = r.at<float>(r.L.skpart);
  float *rstd = r.at<float>(r.L.rstd), *ssq = r.at<float>(r.L.ssq);

  // ------------------------------------------ layers 1..l on every new token ----
  // Two forms of the RMSNorm in front of the QKV and gate/up projections.
  // (a) Fragment-order weights (large batches): the residual epilogue of the O / down GEMM leaves, next to
  //     the fp32 residual stream, ab = bf16(h * gain of the next norm) and the rows' sums of squares; the
  //     next projection reads ab and applies 1/rms as a row factor in its own epilogue.  No pass over h.
  // (b) Otherwise one kernel per norm turns fp32 rows into normed bf16 rows.
  const bool packed = !few_rows && c->have_wpack && T >= 1024;
  const int n_ssq = d / 64;
  if (packed) {
    tm.begin(TC_NORM);
    launch_rmsnorm_rows(h, c->norm1[0], ab, T, d, m.rms_eps, rstd, st);
    tm.end();
  }
  // Few-row batches: a residual GEMM that split K leaves the sum of its splits to the RMSNorm pass that
  // reads the residual rows next (h_pend = number of splits waiting in skp; 1 = none).
  int32_t h_pend = 1;
  for (int j = 0; j < c->l; ++j) {
    if (!packed) {
      tm.begin(TC_NORM);
      launch_rmsnorm_rows(h, c->norm1[j], ab, T, d, m.rms_eps, nullptr, st, skp, h_pend);
      h_pend = 1;
      tm.end();
    }
    if (few_rows) {
      // decode steps and other few-token batches: weights stream once through the skinny kernel (fp32 out),
      // then rotation, rounding and the FP8 absmax in one small pass
      // one launch for [W_Q; W_K; W_V] (through the layer's row-block table): rows of q_dim + 2 kv_dim fp32 columns
      float *q32 = r.at<float>(r.L.qkv32), *k32 = q32 + qd, *v32 = k32 + kvd;
      int32_t fp_splits = 1;
      tm.begin(TC_QKV);
      {
        int32_t ns = 1;   // K splits left to the finishing pass (it reads the fp32 values anyway)
        SkinnyParams sp{ab, T, qd + 2 * kvd, d, nullptr, nullptr, q32, skp, SKINNY_PARTIAL_BYTES, c->qkv_tab[j], &ns};
        if (launch_skinny(sp, EPI_STORE_F32, st)) return fail(SWIFTKV_EHIP, "QKV GEMM launch failed");
        if (ns > 1) { q32 = skp; k32 = q32 + qd; v32 = k32 + kvd; }
        fp_splits = ns;
      }
      QkvFinishParams fp{};
      fp.q32 = q32; fp.k32 = k32; fp.v32 = v32; fp.ld32 = qd + 2 * kvd; fp.n_splits = fp_splits; fp.q = qb; fp.k = kb; fp.v = vb;
      fp.T = T; fp.n_q_heads = m.n_q_heads; fp.n_kv_heads = m.n_kv_heads; fp.head_dim = m.head_dim;
      fp.cos_sin = r.at<float2>(r.L.cos_sin);
      fp.amax = compute_scale ? r.at<uint32_t>(r.L.amax) + (int64_t)j * 2 * m.n_kv_heads : nullptr;
      launch_qkv_finish(fp, st);
      tm.end();
    } else {
      GemmParams g{};
      g.A = ab; g.lda = d; g.M = T; g.N = qd + 2 * kvd; g.K = d;
      g.wtab = c->qkv_tab[j]; g.ldw = d; g.wpack = packed ? c->qkv_pack[j] : nullptr; g.rstd = packed ? rstd : nullptr;
      g.cos_sin = r.at<float2>(r.L.cos_sin);
      g.head_dim = m.head_dim; g.q_dim = qd; g.kv_dim = kvd;
      g.q_out = qb; g.k_out = kb; g.v_out = vb;
      g.first_cache_layer = j;
      g.amax = compute_scale ? r.at<uint32_t>(r.L.amax) : nullptr;
      tm.begin(TC_QKV);
      if (launch_gemm(g, EPI_QKV, 0, st) != 0) return fail(SWIFTKV_EHIP, "QKV GEMM launch failed");
      tm.end();
    }
    {
      CommitParams cp{};
      cp.tiles = (const KVTile *)r.meta(r.L.m_kvtiles); cp.n_tiles = r.L.n_kvtiles;
      cp.n_kv_heads = m.n_kv_heads; cp.head_dim = m.head_dim;
      cp.k_src = kb; cp.v_src = vb; cp.ld_src = kvd;
      cp.cache_k = r.cache_plane(j, 0); cp.cache_v = r.cache_plane(j, 1);
      cp.slots = r.at<int64_t>(r.L.slots);
      cp.fp8 = r.fp8; cp.compute_scale = compute_scale; cp.writeback = r.fp8 && !r.hp.chunked;
      if (r.fp8) {
        cp.amax = r.at<uint32_t>(r.L.amax) + (int64_t)j * 2 * m.n_kv_heads;
        cp.scales = r.layer_scales(j);
        cp.per_token = r.per_token; cp.n_slots = r.n_slots;
      }
      cp.vt = r.hp.chunked ? nullptr : vt; cp.vt_ld = r.L.vt_ld;
      tm.begin(TC_COMMIT);
      if (r.per_token) {
        TokenScaleParams tp{kb, vb, kvd, T, kvd, cp.slots, cp.scales, r.n_slots};
        launch_token_scales(tp, st);
      }
      launch_kv_commit(cp, st);
      tm.end();
      if (r.hp.chunked) {   // cached prefix + the rows just committed -> contiguous K rows and V^T columns
        GatherParams gp{};
        gp.tiles = (const GatherTile *)r.meta(r.L.m_gtiles); gp.n_tiles = r.L.n_gtiles;
        gp.n_kv_heads = m.n_kv_heads; gp.head_dim = m.head_dim;
        gp.cache_k = r.cache_plane(j, 0); gp.cache_v = r.cache_plane(j, 1); gp.fp8 = r.fp8_kind();
        gp.scales = r.fp8 ? r.layer_scales(j) : nullptr;
        gp.block_tables = kv->block_tables; gp.max_blocks_per_seq = kv->max_blocks_per_seq; gp.n_blocks = kv->n_blocks;
        gp.k_dst = r.at<bf16_t>(r.L.kcat); gp.vt = vt; gp.vt_ld = r.L.vt_ld;
        tm.begin(TC_OTHER);
        launch_kv_gather(gp, st);
        tm.end();
      }
    }
    if (r.L.n_qblocks > 0) {
      AttnPrefillParams ap{};
      ap.q = qb; ap.k = r.hp.chunked ? r.at<bf16_t>(r.L.kcat) : kb; ap.vt = vt; ap.vt_ld = r.L.vt_ld; ap.out = ob;
      ap.qblocks = (const QBlock *)r.meta(r.L.m_qblocks); ap.n_qblocks = r.L.n_qblocks;
      ap.sched = r.at<int32_t>(r.L.err) + 4;
      ap.n_q_heads = m.n_q_heads; ap.n_kv_heads = m.n_kv_heads; ap.head_dim = m.head_dim;
      tm.begin(TC_ATTN);
      if (launch_attention_prefill(ap, st) != 0) return fail(SWIFTKV_EHIP, "attention launch failed");
      tm.end();
    }
    if (r.L.n_dec > 0) {  // decode tokens: one query against the paged cache of this layer
      AttnDecodeParams dp{};
      dp.q = qb; dp.out = ob; dp.rows = (const DecodeRow *)r.meta(r.L.m_dec); dp.n_rows = r.L.n_dec;
      dp.n_q_heads = m.n_q_heads; dp.n_kv_heads = m.n_kv_heads; dp.head_dim = m.head_dim;
      dp.cache_k = r.cache_plane(j, 0); dp.cache_v = r.cache_plane(j, 1); dp.fp8 = r.fp8_kind();
      if (r.fp8) { dp.scale_k = r.layer_scales(j); dp.scale_v = dp.scale_k + (r.per_token ? r.n_slots : (int64_t)m.n_kv_heads); }
      dp.block_tables = kv->block_tables; dp.max_blocks_per_seq = kv->max_blocks_per_seq; dp.n_blocks = kv->n_blocks;
      dp.cos_sin = r.at<float2>(r.L.cos_sin); dp.partial = r.at<float>(r.L.partial);
      dp.n_split = pick_split(r.L.n_dec, m.n_kv_heads, r.hp.max_keys_dec);
      tm.begin(TC_OTHER);
      if (launch_attention_decode(dp, st) != 0) return fail(SWIFTKV_EHIP, "decode attention launch failed");
      launch_decode_combine(dp.partial, ob, dp.rows, dp.n_rows, m.n_q_heads, m.head_dim, dp.n_split, st);
      tm.end();
    }
    if (few_rows) {
      tm.begin(TC_O);
      if (tail_gemm(c, ob, T, d, qd, c->wo[j], nullptr, nullptr, h, EPI_RESID, skp, st, &h_pend)) return fail(SWIFTKV_EHIP, "O GEMM launch failed");
      tm.end();
    } else {
      GemmParams g{};
      g.A = ob; g.lda = qd; g.M = T; g.N = d; g.K = qd; g.W = c->wo[j]; g.ldw = qd; g.C = h; g.ldc = d;
      if (packed) { g.wpack = c->wo_pack[j]; g.hb = ab; g.hb_gain = c->norm2[j]; g.ssq = ssq; }
      tm.begin(TC_O);
      if (launch_gemm(g, EPI_RESID, 0, st) != 0) return fail(SWIFTKV_EHIP, "O GEMM launch failed");
      tm.end();
    }
    tm.begin(TC_NORM);
    if (packed) launch_rstd_from_ssq(ssq, n_ssq, rstd, T, d, m.rms_eps, st);
    else { launch_rmsnorm_rows(h, c->norm2[j], ab, T, d, m.rms_eps, nullptr, st, skp, h_pend); h_pend = 1; }
    tm.end();
    if (few_rows) {
      tm.begin(TC_GATEUP);
      if (tail_gemm(c, ab, T, m.ffn, d, c->wgate[j], c->wup[j], c->gu_tab[j], zb, EPI_SWIGLU, skp, st)) return fail(SWIFTKV_EHIP, "gate/up GEMM launch failed");
      tm.end();
      tm.begin(TC_DOWN);
      // (the next reader of h is a norm pass: the next layer's, or the one in front of the later layers' K/V projection)
      if (tail_gemm(c, zb, T, d, m.ffn, c->wdown[j], nullptr, nullptr, h, EPI_RESID, skp, st, (j + 1 < c->l || c->P > 0) ? &h_pend : nullptr))
        return fail(SWIFTKV_EHIP, "down GEMM launch failed");
      tm.end();
    } else {
      {
        GemmParams g{};
        g.A = ab; g.lda = d; g.M = T; g.N = 2 * m.ffn; g.K = d; g.wtab = c->gu_tab[j]; g.ldw = d;
        g.wpack = packed ? c->gu_pack[j] : nullptr; g.rstd = packed ? rstd : nullptr;
        g.C = zb; g.ldc = m.ffn;
        tm.begin(TC_GATEUP);
        if (launch_gemm(g, EPI_SWIGLU, 0, st) != 0) return fail(SWIFTKV_EHIP, "gate/up GEMM launch failed");
        tm.end();
      }
      {
        GemmParams g{};
        g.A = zb; g.lda = m.ffn; g.M = T; g.N = d; g.K = m.ffn; g.W = c->wdown[j]; g.ldw = m.ffn; g.C = h; g.ldc = d;
        if (packed) {   // the next reader of h: the next layer's input norm, or (gain one) the fused K/V projection
          g.wpack = c->down_pack[j]; g.hb = ab; g.hb_gain = j + 1 < c->l ? c->norm1[j + 1] : nullptr; g.ssq = ssq;
        }
        tm.begin(TC_DOWN);
        if (launch_gemm(g, EPI_RESID, 0, st) != 0) return fail(SWIFTKV_EHIP, "down GEMM launch failed");
        tm.end();
      }
      if (packed && (j + 1 < c->l || c->P > 0)) {
        tm.begin(TC_NORM);
        launch_rstd_from_ssq(ssq, n_ssq, rstd, T, d, m.rms_eps, st);
        tm.end();
      }
    }
    if (int e = check_launch("decoder layer")) return e;
  }

  // -------------------------- later layers' K/V from the layer-l output ----
  // operand: the layer-l output rounded to bf16 (the leaders' gains live in the packed weight), 1/rms per row
  if (c->P > 0) {
    if (!packed) {
      tm.begin(TC_NORM);
      launch_rmsnorm_rows(h, nullptr, ab, T, d, m.rms_eps, rstd, st, skp, h_pend);
      h_pend = 1;
      tm.end();
    }
    if (int e = run_fused_kv(r, ab, true, tm)) return e;
  }

  // ----------------------------- last token of every sequence: layers l+1..L ----
  tm.begin(TC_TAIL);
  float *th = r.at<float>(r.L.th);
  bf16_t *ta = r.at<bf16_t>(r.L.ta), *tq = r.at<bf16_t>(r.L.tq), *to = r.at<bf16_t>(r.L.to), *tz = r.at<bf16_t>(r.L.tz);
  launch_gather_rows(h, r.at<int32_t>(r.L.last_rows), th, B, d, st);
  if (c->ee_head) {   // extra head on the layer-l output; the flagged rows' logits replace the final ones below
    launch_rmsnorm_rows(th, c->ee_gain, ta, B, d, m.rms_eps, nullptr, st);
    if (tail_gemm(c, ta, B, m.vocab, d, c->ee_head, nullptr, nullptr, r.at<float>(r.L.ee_logits), EPI_STORE_F32, skp, st))
      return fail(SWIFTKV_EHIP, "early-exit head GEMM failed");
    launch_early_exit_flags(r.at<float>(r.L.ee_logits), B, m.vocab, c->ee_threshold, r.at<int32_t>(r.L.ee_flags), st);
  } else {
    launch_fill_u32(r.at<uint32_t>(r.L.ee_flags), 0, B, st);
  }
  int32_t t_pend = 1;   // K splits of the last residual GEMM waiting for the next norm pass over th
  for (int j = c->l; j < m.n_layers; ++j) {
    const int cl = c->l + (j - c->l) / c->g;
    launch_rmsnorm_rows(th, c->norm1[j], ta, B, d, m.rms_eps, nullptr, st, skp, t_pend);
    if (tail_gemm(c, ta, B, qd, d, c->wq[j], nullptr, nullptr, tq, EPI_STORE_BF16, skp, st)) return fail(SWIFTKV_EHIP, "tail q GEMM failed");
    AttnDecodeParams dp{};
    dp.q = tq; dp.out = to; dp.rows = (const DecodeRow *)r.meta(r.L.m_tail); dp.n_rows = B;
    dp.n_q_heads = m.n_q_heads; dp.n_kv_heads = m.n_kv_heads; dp.head_dim = m.head_dim;
    dp.cache_k = r.cache_plane(cl, 0); dp.cache_v = r.cache_plane(cl, 1); dp.fp8 = r.fp8_kind();
    if (r.fp8) { dp.scale_k = r.layer_scales(cl); dp.scale_v = dp.scale_k + (r.per_token ? r.n_slots : (int64_t)m.n_kv_heads); }
    dp.block_tables = kv->block_tables; dp.max_blocks_per_seq = kv->max_blocks_per_seq; dp.n_blocks = kv->n_blocks;
    dp.cos_sin = r.at<float2>(r.L.cos_sin); dp.partial = r.at<float>(r.L.partial);
    dp.n_split = pick_split(B, m.n_kv_heads, r.hp.max_keys_tail);
    if (launch_attention_decode(dp, st) != 0) return fail(SWIFTKV_EHIP, "tail attention launch failed");
    launch_decode_combine(dp.partial, to, dp.rows, B, m.n_q_heads, m.head_dim, dp.n_split, st);
    if (tail_gemm(c, to, B, d, qd, c->wo[j], nullptr, nullptr, th, EPI_RESID, skp, st, &t_pend)) return fail(SWIFTKV_EHIP, "tail o GEMM failed");
    launch_rmsnorm_rows(th, c->norm2[j], ta, B, d, m.rms_eps, nullptr, st, skp, t_pend);
    if (tail_gemm(c, ta, B, m.ffn, d, c->wgate[j], c->wup[j], c->gu_tab[j], tz, EPI_SWIGLU, skp, st)) return fail(SWIFTKV_EHIP, "tail MLP GEMM failed");
    if (tail_gemm(c, tz, B, d, m.ffn, c->wdown[j], nullptr, nullptr, th, EPI_RESID, skp, st, &t_pend)) return fail(SWIFTKV_EHIP, "tail down GEMM failed");
  }
  launch_rmsnorm_rows(th, c->final_norm, ta, B, d, m.rms_eps, nullptr, st, skp, t_pend);
  if (tail_gemm(c, ta, B, m.vocab, d, c->lm_head, nullptr, nullptr, logits_out, EPI_STORE_F32, skp, st)) return fail(SWIFTKV_EHIP, "LM head GEMM failed");
  if (c->ee_head) launch_early_exit_select(r.at<float>(r.L.ee_logits), r.at<int32_t>(r.L.ee_flags), logits_out, B, m.vocab, st);
  tm.end();
  if (int e = check_launch("tail")) return e;
  c->last = r.L; c->have_last = true;
  return SWIFTKV_OK;
}

int swiftkv_export_plan(swiftkv_ctx *c, const void *workspace, int64_t *slot_mapping, int32_t *positions,
                        int32_t *cu_seqlens, int32_t *last_rows, void *stream) {
  if (!c || !workspace) return fail(SWIFTKV_EINVAL, "null argument");
  if (!c->have_last) return fail(SWIFTKV_EINVAL, "no prefill has run on this ctx");
  const Layout &L = c->last;
  const unsigned char *ws = (const unsigned char *)workspace;
  hipStream_t st = (hipStream_t)stream;
  if (slot_mapping) HIP_TRY(hipMemcpyAsync(slot_mapping, ws + L.slots, L.T * 8, hipMemcpyDeviceToDevice, st));
  if (positions) HIP_TRY(hipMemcpyAsync(positions, ws + L.positions, L.T * 4, hipMemcpyDeviceToDevice, st));
  if (cu_seqlens) HIP_TRY(hipMemcpyAsync(cu_seqlens, ws + L.meta + L.m_cu * 4, (size_t)(L.B + 1) * 4, hipMemcpyDeviceToDevice, st));
  if (last_rows) HIP_TRY(hipMemcpyAsync(last_rows, ws + L.last_rows, (size_t)L.B * 4, hipMemcpyDeviceToDevice, st));
  int32_t flag = 0;
  HIP_TRY(hipMemcpyAsync(&flag, ws + L.err, 4, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (flag & 1) return fail(SWIFTKV_EDATA, "a block table entry was outside [0, n_blocks)");
  if (flag & 2) return fail(SWIFTKV_EDATA, "a token id was outside [0, vocab)");
  return SWIFTKV_OK;
}

int swiftkv_export_hidden(swiftkv_ctx *c, const void *workspace, void *hidden_out, void *stream) {
  if (!c || !workspace || !hidden_out) return fail(SWIFTKV_EINVAL, "null argument");
  if (!c->have_last) return fail(SWIFTKV_EINVAL, "no prefill has run on this ctx");
  const Layout &L = c->last;
  launch_f32_to_bf16((const float *)((const unsigned char *)workspace + L.h), (bf16_t *)hidden_out, (int64_t)L.T * c->cfg.hidden, (hipStream_t)stream);
  return check_launch("hidden export");
}

// ------------------------------------------------------- single operations ----
int swiftkv_op_gemm(const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K, int32_t out_f32,
                    int32_t variant, void *stream) {
  if (!A || !W || !C) return fail(SWIFTKV_EINVAL, "null argument");
  if (M < 1 || N < 16 || K < 8 || (N % 16) || (K % 8)) return fail(SWIFTKV_EINVAL, "need M >= 1, N %% 16 == 0, K %% 8 == 0");
  if (variant != 0 && variant != 1 && variant != 2 && variant != 3 && variant != 14 && variant != 15)
    return fail(SWIFTKV_EINVAL, "variant must be 0, 1, 2, 3, 14 or 15");
  hipStream_t st = (hipStream_t)stream;
  if (variant == 3) {
    if (M > SKINNY_MAX_ROWS) return fail(SWIFTKV_EINVAL, "weight-streaming kernel handles M <= 80");
    SkinnyParams s{(const bf16_t *)A, M, N, K, (const bf16_t *)W, nullptr, C, nullptr, 0, nullptr, nullptr};
    if (launch_skinny(s, out_f32 ? EPI_STORE_F32 : EPI_STORE_BF16, st)) return fail(SWIFTKV_EHIP, "skinny launch failed");
    return check_launch("skinny gemm");
  }
  GemmParams g{};
  g.A = (const bf16_t *)A; g.lda = K; g.M = M; g.N = N; g.K = K; g.W = (const bf16_t *)W; g.ldw = K; g.C = C; g.ldc = N;
  if (launch_gemm(g, out_f32 ? EPI_STORE_F32 : EPI_STORE_BF16, variant, st)) return fail(SWIFTKV_EHIP, "gemm launch failed");
  return check_launch("gemm");
}

int swiftkv_op_gemm_packed(const void *A, const void *W, void *w_packed, void *C, int32_t M, int32_t N, int32_t K, void *stream) {
  if (!A || !W || !w_packed || !C) return fail(SWIFTKV_EINVAL, "null argument");
  if (M < 1024 || N < 256 || K < 256 || (N % 256) || (K % 256)) return fail(SWIFTKV_EINVAL, "need M >= 1024, N %% 256 == 0, K %% 256 == 0");
  hipStream_t st = (hipStream_t)stream;
  launch_pack_w(nullptr, (const bf16_t *)W, K, N, K, 0, (bf16_t *)w_packed, st);
  GemmParams g{};
  g.A = (const bf16_t *)A; g.lda = K; g.M = M; g.N = N; g.K = K; g.W = (const bf16_t *)W; g.ldw = K; g.C = C; g.ldc = N;
  g.wpack = (const bf16_t *)w_packed;
  if (launch_gemm(g, EPI_STORE_BF16, 27, st)) return fail(SWIFTKV_EHIP, "gemm launch failed");
  return check_launch("packed-weight gemm");
}

size_t swiftkv_op_gemm_rows_workspace(int32_t M, int32_t N) {
  if (M < 1 || N < 1) return 0;
  return align_up((size_t)SKINNY_MAX_SPLIT * M * N * 4);
}

int swiftkv_op_gemm_rows(const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K, int32_t out_f32,
                         void *workspace, size_t workspace_bytes, void *stream) {
  if (!A || !W || !C || !workspace) return fail(SWIFTKV_EINVAL, "null argument");
  if (M < 1 || M > SKINNY_MAX_ROWS || N < 16 || K < 8 || (N % 16) || (K % 8))
    return fail(SWIFTKV_EINVAL, "need 1 <= M <= 80, N %% 16 == 0, K %% 8 == 0");
  if (workspace_bytes < swiftkv_op_gemm_rows_workspace(M, N))
    return fail(SWIFTKV_ENOSPC, "workspace has %zu bytes, %zu needed", workspace_bytes, swiftkv_op_gemm_rows_workspace(M, N));
  // (the declared size, not whatever more the caller brought: how K is split depends on the capacity)
  SkinnyParams s{(const bf16_t *)A, M, N, K, (const bf16_t *)W, nullptr, C, (float *)workspace, swiftkv_op_gemm_rows_workspace(M, N), nullptr, nullptr};
  if (launch_skinny(s, out_f32 ? EPI_STORE_F32 : EPI_STORE_BF16, (hipStream_t)stream)) return fail(SWIFTKV_EHIP, "skinny launch failed");
  return check_launch("weight-streaming gemm");
}

// ---- the same kernel for callers that cannot allocate: its scratch is a static device array ----
// 16 splits x 80 rows x 4096 columns of fp32 partial sums (21 MB).  Every GPU the library runs on holds
// its own copy of this array at its own address until the process ends.
constexpr int STATIC_ROWS_MAX_M = SKINNY_MAX_ROWS, STATIC_ROWS_MAX_N = 4096;
constexpr size_t STATIC_SCRATCH_FLOATS = (size_t)SKINNY_MAX_SPLIT * STATIC_ROWS_MAX_M * STATIC_ROWS_MAX_N;
static __device__ __align__(256) float scratch[STATIC_SCRATCH_FLOATS];

// Device address of `scratch` on the current device, looked up once per device (in host code the
// array's name is only a stand-in; kernels must be given this address).
static int static_scratch(float **out) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static float *ptr[MAX_DEV] = {};
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEV) return fail(SWIFTKV_EINVAL, "device index %d out of range", dev);
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(SWIFTKV_EHIP, "hipGetSymbolAddress returned a null address");
    ptr[dev] = (float *)p;
  }
  *out = ptr[dev];
  return 0;
}

int swiftkv_op_gemm_rows_static(const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K, int32_t out_f32,
                                void *stream) {
  if (!A || !W || !C) return fail(SWIFTKV_EINVAL, "null argument");
  if (M < 1 || N < 16 || K < 8 || (N % 16) || (K % 8)) return fail(SWIFTKV_EINVAL, "need M >= 1, N %% 16 == 0, K %% 8 == 0");
  if (M > STATIC_ROWS_MAX_M || N > STATIC_ROWS_MAX_N)
    return fail(SWIFTKV_EINVAL, "M = %d, N = %d beyond the static scratch: at most %d rows and %d columns (use swiftkv_op_gemm_rows "
                "with a workspace for more)", M, N, STATIC_ROWS_MAX_M, STATIC_ROWS_MAX_N);
  float *sp = nullptr;
  if (int e = static_scratch(&sp)) return e;
  // the same scratch capacity as the workspace form declares for this shape: the two then split K alike
  SkinnyParams s{(const bf16_t *)A, M, N, K, (const bf16_t *)W, nullptr, C, sp, swiftkv_op_gemm_rows_workspace(M, N), nullptr, nullptr};
  static_assert(STATIC_SCRATCH_FLOATS * sizeof(float) >= (size_t)SKINNY_MAX_SPLIT * STATIC_ROWS_MAX_M * STATIC_ROWS_MAX_N * 4, "static scratch");
  if (launch_skinny(s, out_f32 ? EPI_STORE_F32 : EPI_STORE_BF16, (hipStream_t)stream)) return fail(SWIFTKV_EHIP, "skinny launch failed");
  return check_launch("weight-streaming gemm (static scratch)");
}

size_t swiftkv_op_attention_workspace(int64_t n_tokens, int32_t n_seqs, int32_t n_kv_heads, int32_t head_dim) {
  const int64_t vt_ld = n_tokens + 64LL * n_seqs;
  return align_up((size_t)n_kv_heads * head_dim * vt_ld * 2) + align_up((size_t)(n_tokens / 128 + n_seqs) * 32) +
         align_up((size_t)(n_tokens / 64 + n_seqs) * 16) + 4096;
}

int swiftkv_op_attention_prefill(const void *q, const void *k, const void *v, void *out, const int32_t *seq_lens,
                                 int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, void *workspace,
                                 size_t workspace_bytes, void *stream) {
  if (!q || !k || !v || !out || !seq_lens || !workspace) return fail(SWIFTKV_EINVAL, "null argument");
  if ((hd != 64 && hd != 128) || Hkv < 1 || Hq % Hkv || (Hkv * hd) % 128 || (Hq * hd) % 128) return fail(SWIFTKV_EINVAL, "bad head shape");
  hipStream_t st = (hipStream_t)stream;
  std::vector<int32_t> qbs, kvt;
  std::vector<std::array<int32_t, 8>> qb_list;
  int64_t row = 0, col = 0;
  for (int b = 0; b < B; ++b) {
    const int n = seq_lens[b];
    if (n < 1) return fail(SWIFTKV_EINVAL, "seq_lens must be >= 1");
    for (int q0 = 0; q0 < n; q0 += 128) qb_list.push_back({(int32_t)(row + q0), q0, n, (int32_t)row, (int32_t)col, (int32_t)(row + n - 1), 0, 0});
    for (int p0 = 0; p0 < n; p0 += 64) kvt.insert(kvt.end(), {(int32_t)(row + p0), std::min(64, n - p0), (int32_t)(col + p0), 0});
    row += n;
    col += (n + 63) / 64 * 64;
  }
  // longest query blocks first (the attention kernel deals them out in that order)
  std::stable_sort(qb_list.begin(), qb_list.end(), [](const std::array<int32_t, 8> &a, const std::array<int32_t, 8> &b) {
    return std::min(a[1] + 128, a[2]) > std::min(b[1] + 128, b[2]);
  });
  for (const auto &e : qb_list) qbs.insert(qbs.end(), e.begin(), e.end());
  const int64_t vt_ld = col;
  size_t o_vt = 0, o_qb = align_up((size_t)Hkv * hd * vt_ld * 2), o_kt = o_qb + align_up(qbs.size() * 4), o_sched = o_kt + align_up(kvt.size() * 4), total = o_sched + 256;
  if (total > workspace_bytes) return fail(SWIFTKV_ENOSPC, "workspace has %zu bytes, %zu needed", workspace_bytes, total);
  unsigned char *ws = (unsigned char *)workspace;
  HIP_TRY(hipMemcpyAsync(ws + o_qb, qbs.data(), qbs.size() * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(hipMemcpyAsync(ws + o_kt, kvt.data(), kvt.size() * 4, hipMemcpyHostToDevice, st));
  CommitParams cp{};
  cp.tiles = (const KVTile *)(ws + o_kt); cp.n_tiles = (int32_t)(kvt.size() / 4); cp.n_kv_heads = Hkv; cp.head_dim = hd;
  cp.k_src = (bf16_t *)k; cp.v_src = (bf16_t *)v; cp.ld_src = (int64_t)Hkv * hd;
  cp.vt = (bf16_t *)(ws + o_vt); cp.vt_ld = vt_ld;
  launch_kv_commit(cp, st);
  AttnPrefillParams ap{};
  ap.q = (const bf16_t *)q; ap.k = (const bf16_t *)k; ap.vt = (const bf16_t *)(ws + o_vt); ap.vt_ld = vt_ld; ap.out = (bf16_t *)out;
  ap.qblocks = (const QBlock *)(ws + o_qb); ap.n_qblocks = (int32_t)(qbs.size() / 8);
  ap.n_q_heads = Hq; ap.n_kv_heads = Hkv; ap.head_dim = hd;
  ap.sched = (int32_t *)(ws + o_sched);
  launch_fill_u32((uint32_t *)(ws + o_sched), 0, 9, st);   // the workspace is the caller's and arrives uninitialised
  if (launch_attention_prefill(ap, st)) return fail(SWIFTKV_EHIP, "attention launch failed");
  if (int e = check_launch("attention")) return e;
  HIP_TRY(hipStreamSynchronize(st));   // the tables above were staged from this call's own (pageable) host vectors
  return SWIFTKV_OK;
}

size_t swiftkv_op_attention_decode_workspace(int32_t n_rows, int32_t n_q_heads, int32_t head_dim) {
  if (n_rows < 1 || n_q_heads < 1 || head_dim < 1) return 0;
  return align_up((size_t)n_rows * sizeof(DecodeRow)) + align_up((size_t)n_rows * n_q_heads * MAX_SPLIT * (head_dim + 2) * 4);
}

int swiftkv_op_attention_decode(const void *q, void *out, const int32_t *n_keys, int32_t n_rows, int32_t Hq, int32_t Hkv,
                                int32_t hd, const void *cache_k, const void *cache_v, int32_t kv_dtype, int32_t scale_mode,
                                const float *scale_k, const float *scale_v, const int32_t *block_tables,
                                int32_t max_blocks_per_seq, int32_t n_blocks, void *workspace, size_t workspace_bytes,
                                void *stream) {
  if (!q || !out || !n_keys || !cache_k || !cache_v || !block_tables || !workspace) return fail(SWIFTKV_EINVAL, "null argument");
  if ((hd != 64 && hd != 128) || Hkv < 1 || Hq % Hkv || n_rows < 1 || n_blocks < 1 || max_blocks_per_seq < 1)
    return fail(SWIFTKV_EINVAL, "bad shape");
  const int R = Hq / Hkv;
  if (R != 1 && R != 2 && R != 4 && R != 8) return fail(SWIFTKV_EINVAL, "query heads per KV head must be 1, 2, 4 or 8");
  const bool fp8 = kv_dtype == SWIFTKV_KV_FP8_E4M3;
  if (!fp8 && kv_dtype != SWIFTKV_KV_BF16) return fail(SWIFTKV_EINVAL, "bad kv dtype");
  if (fp8 && (!scale_k || !scale_v)) return fail(SWIFTKV_EINVAL, "FP8 cache needs scales");
  if (workspace_bytes < swiftkv_op_attention_decode_workspace(n_rows, Hq, hd)) return fail(SWIFTKV_ENOSPC, "workspace too small");
  std::vector<DecodeRow> rows(n_rows);
  int max_keys = 1;
  for (int r = 0; r < n_rows; ++r) {
    if (n_keys[r] < 1 || (n_keys[r] + SKV_BLOCK - 1) / SKV_BLOCK > max_blocks_per_seq) return fail(SWIFTKV_EINVAL, "n_keys[%d] out of range", r);
    rows[r] = DecodeRow{r, r, r, n_keys[r], -1, {0, 0, 0}};
    max_keys = std::max(max_keys, n_keys[r]);
  }
  hipStream_t st = (hipStream_t)stream;
  unsigned char *ws = (unsigned char *)workspace;
  HIP_TRY(hipMemcpyAsync(ws, rows.data(), rows.size() * sizeof(DecodeRow), hipMemcpyHostToDevice, st));
  AttnDecodeParams dp{};
  dp.q = (const bf16_t *)q; dp.out = (bf16_t *)out; dp.rows = (const DecodeRow *)ws; dp.n_rows = n_rows;
  dp.n_q_heads = Hq; dp.n_kv_heads = Hkv; dp.head_dim = hd;
  dp.cache_k = cache_k; dp.cache_v = cache_v;
  dp.fp8 = !fp8 ? 0 : (scale_mode == SWIFTKV_SCALE_PER_TOKEN ? 2 : 1);
  dp.scale_k = scale_k; dp.scale_v = scale_v;
  dp.block_tables = block_tables; dp.max_blocks_per_seq = max_blocks_per_seq; dp.n_blocks = n_blocks;
  dp.partial = (float *)(ws + align_up((size_t)n_rows * sizeof(DecodeRow)));
  dp.n_split = pick_split(n_rows, Hkv, max_keys);
  if (launch_attention_decode(dp, st)) return fail(SWIFTKV_EHIP, "decode attention launch failed");
  launch_decode_combine(dp.partial, dp.out, dp.rows, n_rows, Hq, hd, dp.n_split, st);
  if (int e = check_launch("single-query attention")) return e;
  HIP_TRY(hipStreamSynchronize(st));   // the row table was staged from this call's own (pageable) host vector
  return SWIFTKV_OK;
}

int swiftkv_op_mfma_rate(const void *operands, int32_t iters, void *sink, size_t sink_bytes, double *tflops_out, void *stream) {
  if (!operands || !tflops_out || !sink || iters < 1) return fail(SWIFTKV_EINVAL, "bad argument");
  hipStream_t st = (hipStream_t)stream;
  int dev = 0, n_cu = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  if (sink_bytes < (size_t)n_cu * 256 * 4) return fail(SWIFTKV_ENOSPC, "sink has %zu bytes, %zu needed", sink_bytes, (size_t)n_cu * 256 * 4);
  hipEvent_t e0, e1;
  HIP_TRY(hipEventCreate(&e0));
  HIP_TRY(hipEventCreate(&e1));
  launch_mfma_rate((const bf16_t *)operands, (float *)sink, n_cu, iters / 8 + 1, st);   // warm-up (clocks settle)
  HIP_TRY(hipEventRecord(e0, st));
  launch_mfma_rate((const bf16_t *)operands, (float *)sink, n_cu, iters, st);
  HIP_TRY(hipEventRecord(e1, st));
  HIP_TRY(hipEventSynchronize(e1));
  float ms = 0.f;
  HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (int e = check_launch("mfma rate")) return e;
  *tflops_out = (double)n_cu * 4 * iters * 16 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
  return SWIFTKV_OK;
}

int swiftkv_op_fp8_quantize(const float *x, float scale, uint8_t *codes, int64_t n, void *stream) {
  if (!x || !codes || n < 0) return fail(SWIFTKV_EINVAL, "bad argument");
  launch_fp8_quantize(x, scale, codes, n, (hipStream_t)stream);
  return check_launch("fp8 quantize");
}

}  // extern "C"
