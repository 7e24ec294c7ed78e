// C ABI of libsegattn: argument validation, host mirror of the cache counters, launches.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "segattn_internal.h"

using namespace segattn;

namespace {

#ifndef SEGATTN_DECODE_CHUNK
#define SEGATTN_DECODE_CHUNK 512
#endif
constexpr int kDecodeChunk = SEGATTN_DECODE_CHUNK;  // key rows per split-K workgroup
constexpr unsigned long long kAlign = 256;

unsigned long long align_up(unsigned long long x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool build_problem(const segattn_config *cfg, bool need_cache, Problem &p) {
  if (!cfg || !cfg->kv_policy) return false;
  if (cfg->batch < 1 || cfg->n_kv_heads < 1 || cfg->n_kv_heads > kMaxKvHeads) return false;
  if (cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return false;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return false;
  if (cfg->seg_len < 1 || cfg->tail_len < 0 || cfg->tail_len > cfg->seg_len) return false;
  if ((long long)cfg->seg_len + cfg->tail_len >= (1ll << 30)) return false;
  if (!(cfg->scale >= 0.f) || isinf(cfg->scale)) return false;
  if (!(cfg->rope_theta >= 0.f) || isinf(cfg->rope_theta)) return false;
  if (cfg->prefill_waves != 0 && cfg->prefill_waves != 4 && cfg->prefill_waves != 8) return false;
  if (cfg->item_queues < 0 || cfg->item_queues > 3) return false;
  memset(&p, 0, sizeof(p));
  p.tune_waves = cfg->prefill_waves;
  p.tune_queue = cfg->item_queues;
  p.B = cfg->batch;
  p.Hq = cfg->n_q_heads;
  p.Hkv = cfg->n_kv_heads;
  p.g = p.Hq / p.Hkv;
  p.D = cfg->head_dim;
  p.S = cfg->seg_len;
  p.T = cfg->tail_len;
  p.scale = cfg->scale > 0.f ? cfg->scale : 1.0f / sqrtf((float)p.D);
  p.scale_log2e = p.scale * 1.4426950408889634f;
  p.fp32_math = cfg->fp32_check ? 1 : 0;
  p.out_fp32 = (cfg->fp32_check || cfg->out_fp32) ? 1 : 0;
  int n_past = 0;
  for (int h = 0; h < p.Hkv; ++h) {
    if (cfg->kv_policy[h] > 3) return false;
    p.policy[h] = cfg->kv_policy[h];
    p.past_before[h] = n_past;
    if (p.policy[h] & SEGATTN_PAST) ++n_past;
  }
  p.n_past = n_past;
  int o = 0;
  for (int h = 0; h < p.Hkv; ++h)
    if (p.policy[h] & SEGATTN_PAST) p.order[o++] = h;
  for (int h = 0; h < p.Hkv; ++h)
    if (!(p.policy[h] & SEGATTN_PAST)) p.order[o++] = h;
  if (need_cache && n_past > 0) {
    if (cfg->past_capacity < cfg->seg_len || cfg->past_capacity >= (1ll << 31) - 4096) return false;
  }
  if (need_cache && cfg->retrieved_capacity != 0) {
    if (cfg->retrieved_capacity < 0 || cfg->retrieved_capacity > (1 << 24) || n_past == 0) return false;
    for (int h = 0; h < p.Hkv; ++h)
      if (p.policy[h] == (SEGATTN_TAIL | SEGATTN_PAST)) return false;
  }
  return true;
}

bool build_geom(const segattn_config *cfg, const Problem &p, CacheGeom &g, unsigned long long &total) {
  memset(&g, 0, sizeof(g));
  g.pool_cap = p.n_past ? (unsigned long long)cfg->past_capacity : 0;
  g.ret_cap = cfg->retrieved_capacity;
  g.decode_chunk = kDecodeChunk;
  const unsigned long long past_window = g.ret_cap ? (unsigned long long)g.ret_cap + p.S : g.pool_cap;
  g.ws_splits_past = (int)((past_window + kDecodeChunk - 1) / kDecodeChunk) + 1;
  g.ws_splits_other = (p.T + p.S + kDecodeChunk - 1) / kDecodeChunk + 1;
  g.rows_per_seq = (unsigned long long)p.n_past * g.pool_cap +
                   (unsigned long long)(p.Hkv - p.n_past) * (unsigned long long)(p.T + p.S);
  g.meta_off = 0;
  const unsigned long long meta_bytes = (unsigned long long)p.B * p.Hkv * kMetaInts * 4ull;
  g.ws_off = align_up(meta_bytes);
  const unsigned long long slots = (unsigned long long)p.B * p.g *
                                   ((unsigned long long)p.n_past * g.ws_splits_past +
                                    (unsigned long long)(p.Hkv - p.n_past) * g.ws_splits_other);
  g.kv_off = align_up(g.ws_off + ws_header_bytes(p) + slots * (unsigned long long)ws_slot_floats(p.D) * 4ull);
  g.view_off = align_up(g.kv_off + (unsigned long long)p.B * g.rows_per_seq * 2ull * p.D * 2ull);
  total = g.view_off;
  if (g.ret_cap)
    total += (unsigned long long)p.B * p.n_past * 2ull * (unsigned long long)(g.ret_cap + p.S) * p.D * 2ull;
  // Split-prefix workspace of the segment-by-segment prefill: only where one segment's PAST query
  // blocks (64 rows, up to 4 heads) are at most half as many as the CUs of a 256-CU part -- then
  // the workspace is at most 256 blocks x 64 rows x 4 heads of fp32 output rows (34 MB).
  g.part_max = 1;
  g.part_off = 0;
  if (p.n_past > 0 && g.ret_cap == 0 && p.D == 128 && !p.fp32_math) {
    const int hs = (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1;
    const long long long_wgs = (long long)p.B * p.n_past * (p.g / hs) * ((p.S + (8 / hs) * 32 - 1) / ((8 / hs) * 32));
    long long parts = 256 / long_wgs;
    if (parts > 4) parts = 4;
    if (parts > (long long)(g.pool_cap / 1024)) parts = (long long)(g.pool_cap / 1024);  // >= 1024 rows per piece
    if (parts >= 2) {
      g.part_max = (int)parts;
      g.part_off = align_up(total);
      total = g.part_off + part_ws_bytes(p, g.part_max);
    }
  }
  return total < (1ull << 46);
}

segattn_status hip_status(hipError_t e) { return e == hipSuccess ? SEGATTN_OK : SEGATTN_EHIP; }

// After the runtime has refused a launch or a copy in the middle of a stateful call, earlier
// kernels of that call may already be in the stream, so the device counters can be ahead of the
// host mirror.  The context stops accepting stateful calls until reset / set_lengths.
template <typename Ctx>
segattn_status hip_failed(Ctx *ctx) {
  ctx->ready = false;
  return SEGATTN_EHIP;
}

void fill_inv_freq(double (&t)[64], int D, float theta) {
  for (int i = 0; i < 64; ++i) t[i] = i < D / 2 ? pow((double)theta, -2.0 * i / D) : 0.0;
}

}  // namespace

struct segattn_ctx {
  float rope_theta;
  Problem p;
  CacheGeom g;
  unsigned char *cache;
  bool ready;                       // reset or set_lengths has been enqueued
  std::vector<long long> closed;    // [B] rows in closed segments
  std::vector<int> tail, fill;      // [B]
  std::vector<long long> pool, lo;  // [B*Hkv] (PAST heads)
  std::vector<int> ret;             // [B] rows of the retrieved prefix (retrieval mode)
};

extern "C" {

size_t segattn_cache_bytes(const segattn_config *cfg) {
  Problem p;
  CacheGeom g;
  unsigned long long total;
  if (!build_problem(cfg, true, p) || !build_geom(cfg, p, g, total)) return 0;
  return (size_t)total;
}

segattn_status segattn_create(const segattn_config *cfg, void *cache_dev, size_t cache_bytes,
                              segattn_ctx **out_ctx) {
  if (!out_ctx) return SEGATTN_EINVAL;
  *out_ctx = nullptr;
  Problem p;
  CacheGeom g;
  unsigned long long total;
  if (!build_problem(cfg, true, p) || !build_geom(cfg, p, g, total)) return SEGATTN_EINVAL;
  if (!cache_dev || cache_bytes < total || ((uintptr_t)cache_dev % kAlign)) return SEGATTN_EINVAL;
  segattn_ctx *c = new (std::nothrow) segattn_ctx();
  if (!c) return SEGATTN_EINVAL;
  c->p = p;
  c->rope_theta = cfg->rope_theta;
  c->g = g;
  c->cache = (unsigned char *)cache_dev;
  c->ready = false;
  c->closed.assign(p.B, 0);
  c->tail.assign(p.B, 0);
  c->fill.assign(p.B, 0);
  c->pool.assign((size_t)p.B * p.Hkv, 0);
  c->lo.assign((size_t)p.B * p.Hkv, 0);
  c->ret.assign(p.B, 0);
  *out_ctx = c;
  return SEGATTN_OK;
}

void segattn_destroy(segattn_ctx *ctx) { delete ctx; }

segattn_status segattn_reset(segattn_ctx *ctx, void *stream) {
  if (!ctx) return SEGATTN_EINVAL;
  hipError_t e = launch_cache_reset(ctx->p, ctx->cache, ctx->g, (hipStream_t)stream);
  if (e != hipSuccess) return hip_failed(ctx);
  std::fill(ctx->closed.begin(), ctx->closed.end(), 0);
  std::fill(ctx->tail.begin(), ctx->tail.end(), 0);
  std::fill(ctx->fill.begin(), ctx->fill.end(), 0);
  std::fill(ctx->pool.begin(), ctx->pool.end(), 0);
  std::fill(ctx->lo.begin(), ctx->lo.end(), 0);
  std::fill(ctx->ret.begin(), ctx->ret.end(), 0);
  ctx->ready = true;
  return SEGATTN_OK;
}

segattn_status seg_attn_fwd(segattn_ctx *ctx, const void *q, const void *k, const void *v, int32_t m,
                            void *out, float *lse, void *stream) {
  if (!ctx || !q || !k || !v || !out || !lse || m < 1) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  const Problem &p = ctx->p;
  for (int b = 0; b < p.B; ++b)
    if ((long long)ctx->fill[b] + m > p.S) return SEGATTN_ESTATE;
  PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const unsigned short *)q;
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.out = out;
  a.lse = lse;
  a.cache = ctx->cache;
  a.geom = ctx->g;
  a.n_rows = m;
  a.n_seg = 1;
  a.min_past_prefix = 0;
  if (ctx->g.part_max > 1) {  // fewest prefix rows among the PAST windows: how far their work can be split
    long long least = -1;
    for (int b = 0; b < p.B; ++b)
      for (int h = 0; h < p.Hkv; ++h)
        if (p.policy[h] & SEGATTN_PAST) {
          const size_t i = (size_t)b * p.Hkv + h;
          const long long rows = ctx->pool[i] - ctx->lo[i] + ctx->fill[b];
          if (least < 0 || rows < least) least = rows;
        }
    a.min_past_prefix = least < 0 ? 0 : least;
  }
  return hip_status(launch_prefill(p, a, (hipStream_t)stream));
}

segattn_status seg_attn_fwd_seq(const segattn_config *cfg, const void *q, const void *k, const void *v,
                                int64_t n, void *out, float *lse, void *stream) {
  Problem p;
  if (!build_problem(cfg, false, p)) return SEGATTN_EINVAL;
  if (!q || !k || !v || !out || !lse || n < 1 || n >= (1ll << 31) - 4096) return SEGATTN_EINVAL;
  PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const unsigned short *)q;
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.out = out;
  a.lse = lse;
  a.cache = nullptr;
  a.n_rows = (int)n;
  a.n_seg = (int)((n + p.S - 1) / p.S);
  return hip_status(launch_prefill(p, a, (hipStream_t)stream));
}

segattn_status seg_attn_fwd_varlen(const segattn_config *cfg, const void *q, const void *k, const void *v,
                                   const int32_t *cu_seqlens, int64_t total, int64_t max_seqlen, void *out,
                                   float *lse, void *stream) {
  Problem p;
  if (!build_problem(cfg, false, p)) return SEGATTN_EINVAL;
  if (!q || !k || !v || !out || !lse || !cu_seqlens) return SEGATTN_EINVAL;
  if (max_seqlen < 1 || total < max_seqlen || total >= (1ll << 31) - 4096) return SEGATTN_EINVAL;
  PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const unsigned short *)q;
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.out = out;
  a.lse = lse;
  a.cache = nullptr;
  a.cu_seqlens = cu_seqlens;
  a.total_rows = total;
  a.n_rows = (int)max_seqlen;
  a.n_seg = (int)((max_seqlen + p.S - 1) / p.S);
  return hip_status(launch_prefill(p, a, (hipStream_t)stream));
}

segattn_status segattn_layer_policy(int32_t n_kv_heads, const int32_t *long_heads, int32_t n_long,
                                    int32_t layer_in_l_long, uint8_t *policy_out) {
  if (n_kv_heads < 1 || n_kv_heads > kMaxKvHeads || n_long < 0 || (n_long > 0 && !long_heads) || !policy_out)
    return SEGATTN_EINVAL;
  for (int h = 0; h < n_kv_heads; ++h) policy_out[h] = SEGATTN_TAIL;
  for (int i = 0; i < n_long; ++i) {
    if (long_heads[i] < 0 || long_heads[i] >= n_kv_heads) return SEGATTN_EINVAL;
    policy_out[long_heads[i]] = layer_in_l_long ? SEGATTN_PAST : SEGATTN_SEG;
  }
  return SEGATTN_OK;
}

segattn_status seg_rope_apply(const segattn_config *cfg, void *q, void *k, int64_t rows, const int64_t *pos0,
                              void *stream) {
  Problem p;
  if (!build_problem(cfg, false, p)) return SEGATTN_EINVAL;
  if (!q || !k || rows < 1 || rows >= (1ll << 31) - 4096 || !(cfg->rope_theta > 0.f)) return SEGATTN_EINVAL;
  RopeArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (unsigned short *)q;
  a.k = (unsigned short *)k;
  a.pos0 = (const long long *)pos0;
  a.rows = (int)rows;
  fill_inv_freq(a.inv_freq, p.D, cfg->rope_theta);
  return hip_status(launch_rope_apply(p, a, (hipStream_t)stream));
}

// One row statistic of the backward pass (a float per query head and token row), 256-byte aligned;
// the workspace holds two: delta and -LSE/scale.
static unsigned long long bwd_stat_bytes(const Problem &p, unsigned long long token_rows) {
  return align_up((unsigned long long)p.Hq * token_rows * 4ull);
}

size_t seg_attn_bwd_workspace_bytes(const segattn_config *cfg, int64_t n) {
  Problem p;
  if (!build_problem(cfg, false, p) || n < 1 || n >= (1ll << 31) - 4096) return 0;
  return (size_t)(2ull * bwd_stat_bytes(p, (unsigned long long)p.B * (unsigned long long)n));
}

// Common part of the two whole-sequence backward entry points: `stats` holds the two [B,Hq,n] fp32
// row statistics the kernels keep between them (delta, then -LSE/scale), wherever the caller of
// this function found room for them.
static segattn_status bwd_seq_launch(const Problem &p, const void *q, const void *k, const void *v, const void *out,
                                     const float *lse, const void *dout, int64_t n, void *dq, void *dk, void *dv,
                                     float *stats, void *stream) {
  BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const unsigned short *)q;
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.dout = (const unsigned short *)dout;
  a.out = out;
  a.lse = lse;
  a.delta = stats;
  a.nls = stats + bwd_stat_bytes(p, (unsigned long long)p.B * (unsigned long long)n) / 4;
  a.dq = dq;
  a.dk = dk;
  a.dv = dv;
  a.n = (int)n;
  const hipStream_t st = (hipStream_t)stream;
  if (launch_bwd_delta(p, a, st) != hipSuccess) return SEGATTN_EHIP;
  return hip_status(p.fp32_math ? launch_bwd_fp32(p, a, st) : launch_bwd_mfma(p, a, st));
}

segattn_status seg_attn_bwd_seq(const segattn_config *cfg, const void *q, const void *k, const void *v,
                                const void *out, const float *lse, const void *dout, int64_t n, void *dq,
                                void *dk, void *dv, void *workspace, size_t workspace_bytes, void *stream) {
  Problem p;
  if (!build_problem(cfg, false, p)) return SEGATTN_EINVAL;
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace) return SEGATTN_EINVAL;
  if (n < 1 || n >= (1ll << 31) - 4096) return SEGATTN_EINVAL;
  if (workspace_bytes < seg_attn_bwd_workspace_bytes(cfg, n) || ((uintptr_t)workspace % kAlign))
    return SEGATTN_EINVAL;
  return bwd_seq_launch(p, q, k, v, out, lse, dout, n, dq, dk, dv, (float *)workspace, stream);
}

// ---- the same backward pass for callers that cannot allocate ------------------------------------
// The row statistic lives in an array that is part of the library's device image: one copy per
// GPU, at an address of its own, present from the moment the image is loaded until the process
// ends.  In host code the array's name is only a handle for the runtime; the address kernels and
// copies can use is asked from the runtime once per device (with that device current) and kept.
namespace {
static __device__ __align__(256) unsigned char scratch[SEGATTN_BWD_STATIC_SCRATCH_BYTES];
constexpr int kScratchDevices = 64;

float *static_scratch(hipError_t &err) {
  static std::mutex mu;
  static void *addr[kScratchDevices] = {};
  int dev = -1;
  err = hipGetDevice(&dev);
  if (err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kScratchDevices) {
    err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void *ptr = nullptr;
    err = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (err == hipSuccess && !ptr) err = hipErrorInvalidSymbol;
    if (err != hipSuccess) return nullptr;
    addr[dev] = ptr;
  }
  return (float *)addr[dev];
}
}  // namespace

segattn_status seg_attn_bwd_seq_static(const segattn_config *cfg, const void *q, const void *k, const void *v,
                                       const void *out, const float *lse, const void *dout, int64_t n, void *dq,
                                       void *dk, void *dv, void *stream) {
  Problem p;
  if (!build_problem(cfg, false, p)) return SEGATTN_EINVAL;
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return SEGATTN_EINVAL;
  if (n < 1 || n >= (1ll << 31) - 4096) return SEGATTN_EINVAL;
  // two statistics of B * Hq * n floats must fit the array (checked before anything touches the device)
  if (2ull * bwd_stat_bytes(p, (unsigned long long)p.B * (unsigned long long)n) > (unsigned long long)SEGATTN_BWD_STATIC_SCRATCH_BYTES)
    return SEGATTN_ESCRATCH;
  hipError_t err = hipSuccess;
  float *stats = static_scratch(err);
  if (!stats) {
    (void)hipGetLastError();
    return SEGATTN_EHIP;
  }
  // nothing in the array has to start at zero: the first kernel overwrites every entry that is read
  return bwd_seq_launch(p, q, k, v, out, lse, dout, n, dq, dk, dv, stats, stream);
}

size_t seg_attn_bwd_varlen_workspace_bytes(const segattn_config *cfg, int64_t total) {
  Problem p;
  if (!build_problem(cfg, false, p) || total < 1 || total >= (1ll << 31) - 4096) return 0;
  return (size_t)(2ull * bwd_stat_bytes(p, (unsigned long long)total));
}

segattn_status seg_attn_bwd_varlen(const segattn_config *cfg, const void *q, const void *k, const void *v,
                                   const void *out, const float *lse, const void *dout,
                                   const int32_t *cu_seqlens, int64_t total, int64_t max_seqlen, void *dq,
                                   void *dk, void *dv, void *workspace, size_t workspace_bytes, void *stream) {
  Problem p;
  if (!build_problem(cfg, false, p)) return SEGATTN_EINVAL;
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace || !cu_seqlens)
    return SEGATTN_EINVAL;
  if (max_seqlen < 1 || total < max_seqlen || total >= (1ll << 31) - 4096) return SEGATTN_EINVAL;
  if (workspace_bytes < seg_attn_bwd_varlen_workspace_bytes(cfg, total) || ((uintptr_t)workspace % kAlign))
    return SEGATTN_EINVAL;
  BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const unsigned short *)q;
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.dout = (const unsigned short *)dout;
  a.out = out;
  a.lse = lse;
  a.delta = (float *)workspace;
  a.nls = a.delta + bwd_stat_bytes(p, (unsigned long long)total) / 4;
  a.dq = dq;
  a.dk = dk;
  a.dv = dv;
  a.n = (int)max_seqlen;
  a.cu_seqlens = cu_seqlens;
  a.total = total;
  const hipStream_t st = (hipStream_t)stream;
  if (launch_bwd_delta(p, a, st) != hipSuccess) return SEGATTN_EHIP;
  return hip_status(p.fp32_math ? launch_bwd_fp32(p, a, st) : launch_bwd_mfma(p, a, st));
}

segattn_status seg_kv_commit(segattn_ctx *ctx, const void *k, const void *v, int32_t m, void *stream) {
  if (!ctx || !k || !v || m < 1) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  const Problem &p = ctx->p;
  bool any_full = false;
  for (int b = 0; b < p.B; ++b) {
    if ((long long)ctx->fill[b] + m > p.S) return SEGATTN_ESTATE;
    for (int h = 0; h < p.Hkv; ++h)
      if ((p.policy[h] & SEGATTN_PAST) &&
          ctx->pool[(size_t)b * p.Hkv + h] + ctx->fill[b] + m > (long long)ctx->g.pool_cap)
        return SEGATTN_ECAPACITY;
    any_full |= ctx->fill[b] + m == p.S;
  }
  CopyArgs a;
  memset(&a, 0, sizeof(a));
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.cache = ctx->cache;
  a.geom = ctx->g;
  a.m = m;
  hipError_t e = launch_cache_append(p, a, (hipStream_t)stream);
  if (e == hipSuccess) e = launch_cache_close(p, ctx->cache, ctx->g, m, (hipStream_t)stream);
  if (e != hipSuccess) return hip_failed(ctx);
  (void)any_full;
  for (int b = 0; b < p.B; ++b) {
    ctx->fill[b] += m;
    if (ctx->fill[b] == p.S) {
      ctx->fill[b] = 0;
      ctx->tail[b] = p.T;
      ctx->ret[b] = 0;
      ctx->closed[b] += p.S;
      for (int h = 0; h < p.Hkv; ++h)
        if (p.policy[h] & SEGATTN_PAST) ctx->pool[(size_t)b * p.Hkv + h] += p.S;
    }
  }
  return SEGATTN_OK;
}

segattn_status seg_kv_commit_seq(segattn_ctx *ctx, const void *k, const void *v, int64_t n, void *stream) {
  if (!ctx || !k || !v || n < 1 || n >= (1ll << 31) - 4096) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  const Problem &p = ctx->p;
  for (int b = 0; b < p.B; ++b) {
    if (ctx->fill[b] != 0) return SEGATTN_ESTATE;
    for (int h = 0; h < p.Hkv; ++h)
      if ((p.policy[h] & SEGATTN_PAST) && ctx->pool[(size_t)b * p.Hkv + h] + n > (long long)ctx->g.pool_cap)
        return SEGATTN_ECAPACITY;
  }
  CopyArgs a;
  memset(&a, 0, sizeof(a));
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.cache = ctx->cache;
  a.geom = ctx->g;
  a.m = (int)n;
  if (launch_cache_commit_seq(p, a, (hipStream_t)stream) != hipSuccess) return hip_failed(ctx);
  const long long n_full = n / p.S;
  for (int b = 0; b < p.B; ++b) {
    ctx->fill[b] = (int)(n % p.S);
    if (n_full > 0) {
      ctx->tail[b] = p.T;
      ctx->ret[b] = 0;
      ctx->closed[b] += n_full * p.S;
      for (int h = 0; h < p.Hkv; ++h)
        if (p.policy[h] & SEGATTN_PAST) ctx->pool[(size_t)b * p.Hkv + h] += n_full * p.S;
    }
  }
  return SEGATTN_OK;
}

segattn_status seg_kv_past_append(segattn_ctx *ctx, int32_t kv_head, const void *k, const void *v,
                                  int64_t rows, void *stream) {
  if (!ctx || !k || !v || rows < 1 || kv_head < 0 || kv_head >= ctx->p.Hkv) return SEGATTN_EINVAL;
  const Problem &p = ctx->p;
  if (!(p.policy[kv_head] & SEGATTN_PAST)) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  for (int b = 0; b < p.B; ++b) {
    if (ctx->fill[b] != 0) return SEGATTN_ESTATE;
    if (ctx->pool[(size_t)b * p.Hkv + kv_head] + rows > (long long)ctx->g.pool_cap) return SEGATTN_ECAPACITY;
  }
  CopyArgs a;
  memset(&a, 0, sizeof(a));
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.cache = ctx->cache;
  a.geom = ctx->g;
  a.m = (int)rows;
  a.kv_head = kv_head;
  if (launch_cache_past_append(p, a, (hipStream_t)stream) != hipSuccess) return hip_failed(ctx);
  for (int b = 0; b < p.B; ++b) ctx->pool[(size_t)b * p.Hkv + kv_head] += rows;
  return SEGATTN_OK;
}

segattn_status seg_kv_past_select(segattn_ctx *ctx, const int32_t *idx, int32_t R, void *stream) {
  if (!ctx || R < 0 || (R > 0 && !idx)) return SEGATTN_EINVAL;
  const Problem &p = ctx->p;
  if (ctx->g.ret_cap == 0 || R > ctx->g.ret_cap) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  for (int b = 0; b < p.B; ++b) {
    if (ctx->fill[b] != 0) return SEGATTN_ESTATE;
    for (int h = 0; h < p.Hkv; ++h) {
      const size_t i = (size_t)b * p.Hkv + h;
      if ((p.policy[h] & SEGATTN_PAST) && R > ctx->pool[i] - ctx->lo[i]) return SEGATTN_ECAPACITY;
    }
  }
  SelectArgs a;
  memset(&a, 0, sizeof(a));
  a.idx = idx;
  a.cache = ctx->cache;
  a.geom = ctx->g;
  a.R = R;
  a.rope = ctx->rope_theta > 0.f;
  if (a.rope) fill_inv_freq(a.inv_freq, p.D, ctx->rope_theta);
  if (launch_cache_select(p, a, (hipStream_t)stream) != hipSuccess) return hip_failed(ctx);
  for (int b = 0; b < p.B; ++b) ctx->ret[b] = R;
  return SEGATTN_OK;
}

namespace {
constexpr int kRetrieveCand = 32;
// Pool rows per scoring workgroup.  4096 where that still fills the chip four times over (3
// workgroups per CU); else 1024 -- a last, partly filled round of 1 MB workgroups costs more than
// the extra per-chunk selections; and 512 where even 1024-row chunks are fewer than the CUs (one
// segment's retrieval on a single sequence: the call is then as long as one workgroup's chain
// of tiles, and halving the chain halves it) as long as the merge kernel's fast path still holds
// the lists (256 per head).  The workspace is sized for the smallest chunks.
constexpr int kRetrieveChunkTiny = 512, kRetrieveChunkSmall = 1024, kRetrieveChunkBig = 4096;
int retrieve_chunk_rows(const segattn_ctx *ctx) {
#ifdef SEGATTN_RETRIEVE_CHUNK
  return SEGATTN_RETRIEVE_CHUNK;
#endif
  const Problem &p = ctx->p;
  long long active_big = 0, active_small = 0, longest = 0;
  for (int b = 0; b < p.B; ++b)
    for (int h = 0; h < p.Hkv; ++h) {
      const size_t i = (size_t)b * p.Hkv + h;
      if ((p.policy[h] & SEGATTN_PAST) && ctx->pool[i] > ctx->lo[i]) {
        active_big += (ctx->pool[i] - 1) / kRetrieveChunkBig - ctx->lo[i] / kRetrieveChunkBig + 1;
        active_small += (ctx->pool[i] - 1) / kRetrieveChunkSmall - ctx->lo[i] / kRetrieveChunkSmall + 1;
        if (ctx->pool[i] > longest) longest = ctx->pool[i];
      }
    }
  if (active_big >= 4 * 3 * 256) return kRetrieveChunkBig;
  if (active_small < 256 && (longest + kRetrieveChunkTiny - 1) / kRetrieveChunkTiny <= 256) return kRetrieveChunkTiny;
  return kRetrieveChunkSmall;
}
bool retrieval_layout(const segattn_ctx *ctx, const segattn_retrieval *r, int &nsp, int &n_chunks,
                      unsigned long long &off_val, unsigned long long &off_idx, unsigned long long &total) {
  if (!ctx || !r || ctx->p.n_past == 0) return false;
  if (r->n_queries < 1 || r->pool_window < 1 || r->tail_avg < 1 || r->n_anchors < 1 || r->n_anchors > kRetrieveCand)
    return false;
  if (r->win_before < 0 || r->win_after < 0 || r->win_before > (1 << 20) || r->win_after > (1 << 20)) return false;
  if (ctx->g.pool_cap > (1ull << 20)) return false;
  const long long n_sum = (long long)(r->n_queries + r->pool_window - 1) / r->pool_window + 1;
  if (n_sum * ctx->p.g > 64) return false;
  nsp = (int)((n_sum * ctx->p.g + 31) / 32 * 32);
  n_chunks = (int)((ctx->g.pool_cap + kRetrieveChunkTiny - 1) / kRetrieveChunkTiny);  // the most a call can use
  const unsigned long long heads = (unsigned long long)ctx->p.B * ctx->p.n_past;
  off_val = align_up(heads * nsp * ctx->p.D * 2ull);
  off_idx = align_up(off_val + heads * n_chunks * kRetrieveCand * 4ull);
  total = align_up(off_idx + heads * n_chunks * kRetrieveCand * 4ull);
  return true;
}
}  // namespace

size_t seg_kv_retrieve_workspace_bytes(const segattn_ctx *ctx, const segattn_retrieval *r) {
  int nsp, n_chunks;
  unsigned long long a, b, total;
  return retrieval_layout(ctx, r, nsp, n_chunks, a, b, total) ? (size_t)total : 0;
}

segattn_status seg_kv_retrieve(segattn_ctx *ctx, const segattn_retrieval *r, const void *q_prev, int32_t m,
                               int32_t R, int32_t *idx_out, void *workspace, size_t workspace_bytes,
                               void *stream) {
  int nsp, n_chunks;
  unsigned long long off_val, off_idx, total;
  if (!retrieval_layout(ctx, r, nsp, n_chunks, off_val, off_idx, total)) return SEGATTN_EINVAL;
  if (!q_prev || !idx_out || !workspace || m < 1 || R < 1 || R > (1 << 20)) return SEGATTN_EINVAL;
  if (workspace_bytes < total || ((uintptr_t)workspace % kAlign)) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  const Problem &p = ctx->p;
  for (int b = 0; b < p.B; ++b)
    for (int h = 0; h < p.Hkv; ++h) {
      const size_t i = (size_t)b * p.Hkv + h;
      if ((p.policy[h] & SEGATTN_PAST) && R > ctx->pool[i] - ctx->lo[i]) return SEGATTN_ECAPACITY;
    }
  RetrieveArgs a;
  memset(&a, 0, sizeof(a));
  a.q_prev = (const unsigned short *)q_prev;
  a.cache = ctx->cache;
  a.geom = ctx->g;
  a.summaries = (unsigned short *)workspace;
  a.cand_val = (float *)((unsigned char *)workspace + off_val);
  a.cand_idx = (int *)((unsigned char *)workspace + off_idx);
  a.idx_out = idx_out;
  a.m = m;
  a.R = R;
  a.nsp = nsp;
  a.chunk_rows = retrieve_chunk_rows(ctx);
  long long longest = 1;  // chunks up to the longest pool only
  for (int b = 0; b < p.B; ++b)
    for (int h = 0; h < p.Hkv; ++h)
      if ((p.policy[h] & SEGATTN_PAST) && ctx->pool[(size_t)b * p.Hkv + h] > longest)
        longest = ctx->pool[(size_t)b * p.Hkv + h];
  a.n_chunks = (int)((longest + a.chunk_rows - 1) / a.chunk_rows);
  if (a.n_chunks > n_chunks) return SEGATTN_EINVAL;
  a.n_queries = r->n_queries;
  a.pool_window = r->pool_window;
  a.tail_avg = r->tail_avg;
  a.n_anchors = r->n_anchors;
  a.win_before = r->win_before;
  a.win_after = r->win_after;
  return hip_status(launch_retrieve(p, a, (hipStream_t)stream));
}

// ---- stateless retrieval mode: the whole prompt at once ---------------------------------------
namespace {
// Problem of a stateless retrieval-mode call: at least one PAST head, none with TAIL as well
// (Eq. 13 gives a long-range head its retrieved prefix and no tail), 1 <= R <= S so that every
// segment after the first has R pool rows to choose from.
bool build_retrieval_problem(const segattn_config *cfg, int64_t n, int32_t R, Problem &p, int &n_seg) {
  if (!build_problem(cfg, false, p)) return false;
  if (n < 1 || n >= (1ll << 31) - 4096 || R < 1 || R > p.S || p.n_past == 0) return false;
  for (int h = 0; h < p.Hkv; ++h)
    if (p.policy[h] == (SEGATTN_TAIL | SEGATTN_PAST)) return false;
  n_seg = (int)((n + p.S - 1) / p.S);
  return true;
}
constexpr int kRetrieveSeqChunk = 1024;  // pool rows per scoring workgroup of the whole-prompt form
bool retrieval_seq_layout(const Problem &p, const segattn_retrieval *r, int64_t n, int n_seg, int &nsp, int &n_chunks,
                          unsigned long long &off_val, unsigned long long &off_idx, unsigned long long &total) {
  if (!r || r->n_queries < 1 || r->pool_window < 1 || r->tail_avg < 1 || r->n_anchors < 1 || r->n_anchors > kRetrieveCand)
    return false;
  if (r->win_before < 0 || r->win_after < 0 || r->win_before > (1 << 20) || r->win_after > (1 << 20)) return false;
  if (n > (1ll << 20)) return false;
  const long long n_sum = (long long)(r->n_queries + r->pool_window - 1) / r->pool_window + 1;
  if (n_sum * p.g > 64) return false;
  nsp = (int)((n_sum * p.g + 31) / 32 * 32);
  const long long longest = (long long)(n_seg - 1) * p.S;  // pool of the last segment
  n_chunks = (int)((longest + kRetrieveSeqChunk - 1) / kRetrieveSeqChunk);
  if (n_chunks < 1) n_chunks = 1;
  const unsigned long long heads = (unsigned long long)p.B * n_seg * p.n_past;
  off_val = align_up(heads * nsp * p.D * 2ull);
  off_idx = align_up(off_val + heads * n_chunks * kRetrieveCand * 4ull);
  total = align_up(off_idx + heads * n_chunks * kRetrieveCand * 4ull);
  return true;
}
}  // namespace

size_t seg_kv_retrieve_seq_workspace_bytes(const segattn_config *cfg, const segattn_retrieval *r, int64_t n) {
  Problem p;
  int n_seg, nsp, n_chunks;
  unsigned long long a, b, total;
  if (!build_retrieval_problem(cfg, n, 1, p, n_seg) || !retrieval_seq_layout(p, r, n, n_seg, nsp, n_chunks, a, b, total))
    return 0;
  return (size_t)total;
}

segattn_status seg_kv_retrieve_seq(const segattn_config *cfg, const segattn_retrieval *r, const void *q, const void *k,
                                   int64_t n, int32_t R, int32_t *idx_out, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  Problem p;
  int n_seg, nsp, n_chunks;
  unsigned long long off_val, off_idx, total;
  if (!build_retrieval_problem(cfg, n, R, p, n_seg) ||
      !retrieval_seq_layout(p, r, n, n_seg, nsp, n_chunks, off_val, off_idx, total))
    return SEGATTN_EINVAL;
  if (!q || !k || !idx_out || !workspace || workspace_bytes < total || ((uintptr_t)workspace % kAlign)) return SEGATTN_EINVAL;
  RetrieveArgs a;
  memset(&a, 0, sizeof(a));
  a.q_prev = (const unsigned short *)q;
  a.k_seq = (const unsigned short *)k;
  a.n_rows = (int)n;
  a.n_seg = n_seg;
  a.summaries = (unsigned short *)workspace;
  a.cand_val = (float *)((unsigned char *)workspace + off_val);
  a.cand_idx = (int *)((unsigned char *)workspace + off_idx);
  a.idx_out = idx_out;
  a.m = p.S;
  a.R = R;
  a.nsp = nsp;
  a.chunk_rows = kRetrieveSeqChunk;
  a.n_chunks = n_chunks;
  a.n_queries = r->n_queries;
  a.pool_window = r->pool_window;
  a.tail_avg = r->tail_avg;
  a.n_anchors = r->n_anchors;
  a.win_before = r->win_before;
  a.win_after = r->win_after;
  return hip_status(launch_retrieve(p, a, (hipStream_t)stream));
}

size_t seg_attn_fwd_seq_retrieved_workspace_bytes(const segattn_config *cfg, int64_t n, int32_t R) {
  Problem p;
  int n_seg;
  if (!build_retrieval_problem(cfg, n, R, p, n_seg)) return 0;
  return (size_t)(2ull * align_up((unsigned long long)p.B * n_seg * p.n_past * (unsigned long long)R * p.D * 2ull));
}

segattn_status seg_attn_fwd_seq_retrieved(const segattn_config *cfg, const void *q, const void *k, const void *v,
                                          int64_t n, const int32_t *idx, int32_t R, void *workspace,
                                          size_t workspace_bytes, void *out, float *lse, void *stream) {
  Problem p;
  int n_seg;
  if (!build_retrieval_problem(cfg, n, R, p, n_seg)) return SEGATTN_EINVAL;
  if (!q || !k || !v || !idx || !out || !lse || !workspace || ((uintptr_t)workspace % kAlign)) return SEGATTN_EINVAL;
  if (workspace_bytes < seg_attn_fwd_seq_retrieved_workspace_bytes(cfg, n, R)) return SEGATTN_EINVAL;
  const unsigned long long half = align_up((unsigned long long)p.B * n_seg * p.n_past * (unsigned long long)R * p.D * 2ull);
  GatherSeqArgs g;
  memset(&g, 0, sizeof(g));
  g.k = (const unsigned short *)k;
  g.v = (const unsigned short *)v;
  g.idx = idx;
  g.ret_k = (unsigned short *)workspace;
  g.ret_v = (unsigned short *)((unsigned char *)workspace + half);
  g.n = (int)n;
  g.n_seg = n_seg;
  g.R = R;
  g.rope = cfg->rope_theta > 0.f;
  if (g.rope) fill_inv_freq(g.inv_freq, p.D, cfg->rope_theta);
  if (launch_gather_seq(p, g, (hipStream_t)stream) != hipSuccess) return SEGATTN_EHIP;
  PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const unsigned short *)q;
  a.k = (const unsigned short *)k;
  a.v = (const unsigned short *)v;
  a.out = out;
  a.lse = lse;
  a.cache = nullptr;
  a.n_rows = (int)n;
  a.n_seg = n_seg;
  a.ret_k = g.ret_k;
  a.ret_v = g.ret_v;
  a.ret_R = R;
  return hip_status(launch_prefill(p, a, (hipStream_t)stream));
}

// n_oldest >= 0 with keep < 0: hide that many more rows; keep >= 0: hide what exceeds `keep`
// visible rows.  The host mirror follows the device counters.
static segattn_status evict_rows(segattn_ctx *ctx, int32_t kv_head, int64_t n_oldest, int64_t keep, void *stream) {
  if (!ctx || kv_head < 0 || kv_head >= ctx->p.Hkv) return SEGATTN_EINVAL;
  const Problem &p = ctx->p;
  if (!(p.policy[kv_head] & SEGATTN_PAST)) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  if (launch_cache_evict(p, ctx->cache, ctx->g, kv_head, n_oldest, keep, (hipStream_t)stream) != hipSuccess)
    return hip_failed(ctx);
  for (int b = 0; b < p.B; ++b) {
    const size_t i = (size_t)b * p.Hkv + kv_head;
    long long limit = ctx->pool[i];
    long long n = n_oldest;
    if (keep >= 0) n = limit - ctx->lo[i] > keep ? limit - ctx->lo[i] - keep : 0;
    if (p.policy[kv_head] & SEGATTN_TAIL) limit -= ctx->tail[b];
    // at most the rows still visible below the limit (n may be anything up to INT64_MAX)
    const long long room = limit > ctx->lo[i] ? limit - ctx->lo[i] : 0;
    ctx->lo[i] += n < room ? n : room;
  }
  return SEGATTN_OK;
}

segattn_status seg_kv_past_evict(segattn_ctx *ctx, int32_t kv_head, int64_t n_oldest, void *stream) {
  if (n_oldest < 0) return SEGATTN_EINVAL;
  return evict_rows(ctx, kv_head, n_oldest, -1, stream);
}

segattn_status seg_kv_past_keep_recent(segattn_ctx *ctx, int32_t kv_head, int64_t max_rows, void *stream) {
  if (max_rows < 0) return SEGATTN_EINVAL;
  return evict_rows(ctx, kv_head, 0, max_rows, stream);
}

segattn_status seg_kv_lengths(const segattn_ctx *ctx, int64_t *past, int32_t *tail, int32_t *seg_fill) {
  if (!ctx) return SEGATTN_EINVAL;
  const Problem &p = ctx->p;
  for (int b = 0; b < p.B; ++b) {
    if (tail) tail[b] = ctx->tail[b];
    if (seg_fill) seg_fill[b] = ctx->fill[b];
    if (past)
      for (int h = 0; h < p.Hkv; ++h) {
        const size_t i = (size_t)b * p.Hkv + h;
        past[i] = (p.policy[h] & SEGATTN_PAST) ? ctx->pool[i] - ctx->lo[i] : 0;
      }
  }
  return SEGATTN_OK;
}

segattn_status seg_kv_set_lengths(segattn_ctx *ctx, const int64_t *closed_rows, const int32_t *tail,
                                  const int32_t *seg_fill, void *stream) {
  if (!ctx || !closed_rows || !tail || !seg_fill) return SEGATTN_EINVAL;
  const Problem &p = ctx->p;
  for (int b = 0; b < p.B; ++b) {
    if (closed_rows[b] < 0 || closed_rows[b] % p.S) return SEGATTN_EINVAL;
    if (seg_fill[b] < 0 || seg_fill[b] >= p.S) return SEGATTN_EINVAL;
    if (ctx->g.ret_cap && seg_fill[b] != 0) return SEGATTN_EINVAL;
    if (tail[b] < 0 || tail[b] > p.T || tail[b] > closed_rows[b]) return SEGATTN_EINVAL;
    if (p.n_past && closed_rows[b] + seg_fill[b] > (long long)ctx->g.pool_cap) return SEGATTN_ECAPACITY;
  }
  // The counters are written by a kernel that takes the lengths by value (a chunk of sequences
  // per launch): nothing the stream still has to read lives in host memory after the call.
  for (int b0 = 0; b0 < p.B; b0 += kLengthsChunk) {
    LengthsArgs la;
    memset(&la, 0, sizeof(la));
    la.b0 = b0;
    la.count = p.B - b0 < kLengthsChunk ? p.B - b0 : kLengthsChunk;
    for (int i = 0; i < la.count; ++i) {
      la.closed[i] = (int)closed_rows[b0 + i];
      la.tail[i] = tail[b0 + i];
      la.fill[i] = seg_fill[b0 + i];
    }
    if (launch_cache_set_lengths(p, ctx->cache, ctx->g, la, (hipStream_t)stream) != hipSuccess) return hip_failed(ctx);
  }
  for (int b = 0; b < p.B; ++b) {
    ctx->closed[b] = closed_rows[b];
    ctx->tail[b] = tail[b];
    ctx->fill[b] = seg_fill[b];
    ctx->ret[b] = 0;
    for (int h = 0; h < p.Hkv; ++h) {
      ctx->pool[(size_t)b * p.Hkv + h] = (p.policy[h] & SEGATTN_PAST) ? closed_rows[b] : 0;
      ctx->lo[(size_t)b * p.Hkv + h] = 0;
    }
  }
  ctx->ready = true;
  return SEGATTN_OK;
}

segattn_status segattn_cache_span(const segattn_ctx *ctx, int32_t b, int32_t kv_head, size_t *k_off,
                                  size_t *v_off, int64_t *cap_rows) {
  if (!ctx || b < 0 || b >= ctx->p.B || kv_head < 0 || kv_head >= ctx->p.Hkv) return SEGATTN_EINVAL;
  if (k_off) *k_off = (size_t)k_block_off(ctx->p, ctx->g, b, kv_head);
  if (v_off) *v_off = (size_t)v_block_off(ctx->p, ctx->g, b, kv_head);
  if (cap_rows) *cap_rows = (int64_t)head_cap(ctx->p, ctx->g, kv_head);
  return SEGATTN_OK;
}

size_t segattn_resident_bytes(const segattn_ctx *ctx) {
  if (!ctx) return 0;
  const Problem &p = ctx->p;
  unsigned long long rows = 0;
  for (int b = 0; b < p.B; ++b)
    for (int h = 0; h < p.Hkv; ++h) {
      if (p.policy[h] & SEGATTN_PAST)
        rows += ctx->pool[(size_t)b * p.Hkv + h] + ctx->fill[b] +
                (ctx->g.ret_cap ? ctx->ret[b] + ctx->fill[b] : 0);
      else rows += ((p.policy[h] & SEGATTN_TAIL) ? ctx->tail[b] : 0) + ctx->fill[b];
    }
  return (size_t)(rows * 2ull * p.D * 2ull);
}

segattn_status seg_attn_decode(segattn_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                               void *out, float *lse, void *stream) {
  if (!ctx || !q || !k_new || !v_new || !out || !lse) return SEGATTN_EINVAL;
  if (!ctx->ready) return SEGATTN_ESTATE;
  const Problem &p = ctx->p;
  long long total_rows = 0;
  bool any_full = false;
  for (int b = 0; b < p.B; ++b) {
    for (int h = 0; h < p.Hkv; ++h) {
      const size_t i = (size_t)b * p.Hkv + h;
      long long win;
      if (p.policy[h] & SEGATTN_PAST) {
        if (ctx->pool[i] + ctx->fill[b] + 1 > (long long)ctx->g.pool_cap) return SEGATTN_ECAPACITY;
        win = (ctx->g.ret_cap ? ctx->ret[b] : ctx->pool[i] - ctx->lo[i]) + ctx->fill[b] + 1;
      } else {
        win = ((p.policy[h] & SEGATTN_TAIL) ? ctx->tail[b] : 0) + ctx->fill[b] + 1;
      }
      total_rows += win;
    }
    any_full |= ctx->fill[b] + 1 == p.S;
  }
  const hipStream_t st = (hipStream_t)stream;
  CopyArgs ca;
  memset(&ca, 0, sizeof(ca));
  ca.k = (const unsigned short *)k_new;
  ca.v = (const unsigned short *)v_new;
  ca.cache = ctx->cache;
  ca.geom = ctx->g;
  ca.m = 1;
  if (launch_cache_decode_append(p, ca, st) != hipSuccess) return hip_failed(ctx);
  DecodeArgs da;
  memset(&da, 0, sizeof(da));
  da.q = (const unsigned short *)q;
  da.k_new = ca.k;
  da.v_new = ca.v;
  da.out = out;
  da.lse = lse;
  da.cache = ctx->cache;
  da.geom = ctx->g;
  da.total_rows = total_rows;
  if (launch_decode(p, da, p.B, st) != hipSuccess) return hip_failed(ctx);
  if (any_full && launch_cache_close(p, ctx->cache, ctx->g, 0, st) != hipSuccess) return hip_failed(ctx);
  for (int b = 0; b < p.B; ++b) {
    ctx->fill[b] += 1;
    if (ctx->fill[b] == p.S) {
      ctx->fill[b] = 0;
      ctx->tail[b] = p.T;
      ctx->ret[b] = 0;
      ctx->closed[b] += p.S;
      for (int h = 0; h < p.Hkv; ++h)
        if (p.policy[h] & SEGATTN_PAST) ctx->pool[(size_t)b * p.Hkv + h] += p.S;
    }
  }
  return SEGATTN_OK;
}

segattn_status segattn_bandwidth_probe(void *buf, size_t bytes, int32_t mode, void *sink, void *stream) {
  if (!buf || !sink || bytes < 16 || ((uintptr_t)buf % 16) || (mode != 0 && mode != 1)) return SEGATTN_EINVAL;
  return hip_status(launch_probe(buf, (long long)bytes, mode, sink, (hipStream_t)stream));
}

segattn_status segattn_clock_probe(uint32_t microseconds, uint64_t *counts, int32_t *wall_clock_khz, void *stream) {
  static_assert(SEGATTN_CLOCK_PROBE_WAVES == kClockProbeWaves, "header and kernel disagree");
  if (!counts || ((uintptr_t)counts % 8) || !wall_clock_khz || microseconds == 0 || microseconds > 10000000u)
    return SEGATTN_EINVAL;
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess ||
      khz <= 0)
    return SEGATTN_EHIP;
  *wall_clock_khz = khz;
  const unsigned long long ticks = (unsigned long long)microseconds * (unsigned long long)khz / 1000ull;
  return hip_status(launch_clock_probe(ticks > 0 ? ticks : 1, (unsigned long long *)counts, (hipStream_t)stream));
}

segattn_status segattn_mfma_probe(int32_t iterations, int32_t operands, void *sink, int64_t *flops, void *stream) {
  if (!sink || ((uintptr_t)sink % 4) || !flops || iterations < 1 || iterations > 10000000 || (operands != 0 && operands != 1))
    return SEGATTN_EINVAL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return SEGATTN_EHIP;
  const int workgroups = 2 * cus;
  *flops = (int64_t)workgroups * 4 * (int64_t)iterations * kMfmaProbeFlopsPerWaveIter;
  return hip_status(launch_mfma_probe(iterations, operands, workgroups, (float *)sink, (hipStream_t)stream));
}

const char *segattn_strerror(segattn_status st) {
  switch (st) {
    case SEGATTN_OK: return "ok";
    case SEGATTN_EINVAL: return "invalid argument or unsupported configuration";
    case SEGATTN_ECAPACITY: return "past pool capacity exceeded";
    case SEGATTN_ESTATE: return "call not valid in the current cache state";
    case SEGATTN_EHIP: return "HIP runtime error";
    case SEGATTN_ESCRATCH: return "problem too large for the library's built-in scratch buffer";
  }
  return "unknown status";
}

const char *segattn_version(void) { return "segattn 0.1 gfx950"; }

}  // extern "C"
