// Cross-segment state of libsegattn (Sec. 3.4): the carried KV tail C_i of local heads and the
// append-only past pool of long-range heads, kept in one caller-owned arena.  All kernels
// here are plain copies (HBM-bound) plus the per-(sequence, head) counters they maintain:
//   counters[b][h] = { pool rows, tail rows, open-segment rows, first visible pool row,
//                      rows of the retrieved prefix }.
// In retrieval mode (Sec. 3.4 "Long-Range Channel", Appendix D "Output") a long-range head
// attends to R gathered pool rows plus its own segment: cache_select_kernel gathers the rows into
// the head's attention view, and every row appended to the open segment is mirrored there.
// The host keeps a mirror of the counters for validation; the device copy is only ever
// changed by these kernels, in stream order, so a sequence of calls can be graph-captured.
#include <math.h>

#include "segattn_internal.h"

namespace segattn {

// Turn 8 channel pairs (lo: channels i0..i0+7, hi: their partners i0+D/2..) by `delta` positions.
__device__ inline void rerotate8(uint4 &lo, uint4 &hi, double delta, const double *inv_freq, int i0) {
  unsigned *lw = (unsigned *)&lo, *hw = (unsigned *)&hi;
  const double two_pi = 6.283185307179586476925286766559;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    unsigned lo_out = 0, hi_out = 0;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float x = __uint_as_float(e ? (lw[w] & 0xffff0000u) : (lw[w] << 16));
      const float y = __uint_as_float(e ? (hw[w] & 0xffff0000u) : (hw[w] << 16));
      const double ang = delta * inv_freq[i0 + 2 * w + e];
      float sn, cs;
      sincosf((float)(ang - two_pi * rint(ang / two_pi)), &sn, &cs);
      const __bf16 ya = (__bf16)(x * cs - y * sn), yb = (__bf16)(x * sn + y * cs);
      lo_out |= (unsigned)__builtin_bit_cast(unsigned short, ya) << (16 * e);
      hi_out |= (unsigned)__builtin_bit_cast(unsigned short, yb) << (16 * e);
    }
    lw[w] = lo_out;
    hw[w] = hi_out;
  }
}

__device__ inline int *meta_of(unsigned char *cache, const CacheGeom &g, const Problem &p, int b, int h) {
  return (int *)(cache + g.meta_off) + ((long long)b * p.Hkv + h) * kMetaInts;
}

__global__ void cache_reset_kernel(const Problem p, unsigned char *cache, const CacheGeom g) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < p.B * p.Hkv * kMetaInts) ((int *)(cache + g.meta_off))[i] = 0;
}

// Rows k,v [B,m,Hkv,D] -> open segment of every (b,h).  grid = (row chunks, B*Hkv).
// A non-PAST head whose whole segment arrives in one call (fill = 0, m = S) keeps only the
// last T rows, written straight into the tail slots; everything else of it is dropped.
template <int D>
__global__ __launch_bounds__(256) void cache_append_kernel(const Problem p, const CopyArgs a) {
  constexpr int CPR = D / 8;  // 16-byte chunks per row
  const int b = blockIdx.y / p.Hkv, h = blockIdx.y % p.Hkv;
  const int *meta = meta_of(a.cache, a.geom, p, b, h);
  const int fill = meta[META_FILL];
  const bool past = p.policy[h] & SEGATTN_PAST;
  int src0 = 0, dst0, n = a.m;
  if (past) {
    dst0 = meta[META_POOL] + fill;
  } else if (fill == 0 && a.m == p.S) {
    src0 = p.S - p.T;
    n = p.T;
    dst0 = 0;
  } else {
    dst0 = p.T + fill;
  }
  const uint4 *ks = (const uint4 *)(a.k + ((long long)b * a.m * p.Hkv + h) * D);
  const uint4 *vs = (const uint4 *)(a.v + ((long long)b * a.m * p.Hkv + h) * D);
  uint4 *kd = (uint4 *)(a.cache + k_block_off(p, a.geom, b, h));
  uint4 *vd = (uint4 *)(a.cache + v_block_off(p, a.geom, b, h));
  const long long src_stride = (long long)p.Hkv * CPR;
  const int rows_per_block = 256 / CPR * 8;
  const int r_begin = blockIdx.x * rows_per_block;
  const int r_end = min(n, r_begin + rows_per_block);
  const int c = threadIdx.x % CPR;
  uint4 *km = nullptr, *vm = nullptr;  // mirror of the open segment in the attention view
  if (uses_view(p, a.geom, h)) {
    km = (uint4 *)(a.cache + view_k_off(p, a.geom, b, h)) + (long long)(a.geom.ret_cap + fill) * CPR;
    vm = (uint4 *)(a.cache + view_v_off(p, a.geom, b, h)) + (long long)(a.geom.ret_cap + fill) * CPR;
  }
  for (int r = r_begin + threadIdx.x / CPR; r < r_end; r += 256 / CPR) {
    const uint4 kx = ks[(long long)(src0 + r) * src_stride + c];
    const uint4 vx = vs[(long long)(src0 + r) * src_stride + c];
    kd[(long long)(dst0 + r) * CPR + c] = kx;
    vd[(long long)(dst0 + r) * CPR + c] = vx;
    if (km) {
      km[(long long)r * CPR + c] = kx;
      vm[(long long)r * CPR + c] = vx;
    }
  }
}

// Close the open segment of every (b,h) whose fill reaches S after adding `add` rows:
// tail <- last T rows of the segment (non-PAST heads), pool += S (PAST heads), fill <- 0; in
// retrieval mode the retrieved prefix belonged to the segment just closed and is dropped.
// One workgroup per (b,h): it alone reads and writes that head's counters.
template <int D>
__global__ __launch_bounds__(256) void cache_close_kernel(const Problem p, unsigned char *cache,
                                                         const CacheGeom g, const int add) {
  constexpr int CPR = D / 8;
  const int b = blockIdx.x / p.Hkv, h = blockIdx.x % p.Hkv;
  int *meta = meta_of(cache, g, p, b, h);
  const int fill_old = meta[META_FILL], pool = meta[META_POOL];
  __syncthreads();
  const int fill = fill_old + add;
  const bool past = p.policy[h] & SEGATTN_PAST;
  if (fill < p.S) {
    if (threadIdx.x == 0) meta[META_FILL] = fill;
    return;
  }
  if (!past && p.T > 0 && !(fill_old == 0 && add == p.S)) {
    uint4 *kd = (uint4 *)(cache + k_block_off(p, g, b, h));
    uint4 *vd = (uint4 *)(cache + v_block_off(p, g, b, h));
    const long long n = (long long)p.T * CPR, src = (long long)p.S * CPR;  // rows [S, S+T) -> [0, T)
    for (long long i = threadIdx.x; i < n; i += 256) {
      kd[i] = kd[src + i];
      vd[i] = vd[src + i];
    }
  }
  if (threadIdx.x == 0) {
    meta[META_FILL] = 0;
    meta[META_TAIL] = p.T;
    if (past) meta[META_POOL] = pool + p.S;
    meta[META_RET] = 0;
  }
}

// Whole prompt at once: rows k,v [B,n,Hkv,D] of a sequence whose open segment is empty -> the state
// n/S commits of S rows and one of n%S rows would leave.  PAST heads: every row goes to the pool
// (whole segments, then the open one behind them).  Other heads: the last T rows of the last whole
// segment become the tail, the n%S open rows follow it.  The open rows are mirrored into the
// attention view in retrieval mode.  grid = (row chunks, B*Hkv); counters: cache_commit_seq_meta.
template <int D>
__global__ __launch_bounds__(256) void cache_commit_seq_kernel(const Problem p, const CopyArgs a) {
  constexpr int CPR = D / 8;
  const int b = blockIdx.y / p.Hkv, h = blockIdx.y % p.Hkv;
  const int *meta = meta_of(a.cache, a.geom, p, b, h);
  const bool past = p.policy[h] & SEGATTN_PAST;
  const int n = a.m, n_full = n / p.S, open = n % p.S, closed_rows = n_full * p.S;
  const int tail_rows = (!past && n_full > 0) ? p.T : 0;
  // virtual rows of this head: [0, head_rows): PAST: source rows 0..n-1 -> pool + r;
  // otherwise: tail rows (source closed_rows - T + r -> r), then open rows (source closed_rows + r' -> T + r')
  const int head_rows = past ? n : tail_rows + open;
  const int pool = meta[META_POOL];
  const uint4 *ks = (const uint4 *)(a.k + ((long long)b * n * p.Hkv + h) * D);
  const uint4 *vs = (const uint4 *)(a.v + ((long long)b * n * p.Hkv + h) * D);
  uint4 *kd = (uint4 *)(a.cache + k_block_off(p, a.geom, b, h));
  uint4 *vd = (uint4 *)(a.cache + v_block_off(p, a.geom, b, h));
  uint4 *km = nullptr, *vm = nullptr;
  if (uses_view(p, a.geom, h)) {
    km = (uint4 *)(a.cache + view_k_off(p, a.geom, b, h)) + (long long)a.geom.ret_cap * CPR;
    vm = (uint4 *)(a.cache + view_v_off(p, a.geom, b, h)) + (long long)a.geom.ret_cap * CPR;
  }
  const long long src_stride = (long long)p.Hkv * CPR;
  const int rows_per_block = 256 / CPR * 8;
  const int r_begin = blockIdx.x * rows_per_block;
  const int r_end = min(head_rows, r_begin + rows_per_block);
  const int c = threadIdx.x % CPR;
  for (int r = r_begin + threadIdx.x / CPR; r < r_end; r += 256 / CPR) {
    int src, dst;
    if (past) {
      src = r;
      dst = pool + r;
    } else if (r < tail_rows) {
      src = closed_rows - p.T + r;
      dst = r;
    } else {
      src = closed_rows + (r - tail_rows);
      dst = p.T + (r - tail_rows);
    }
    const uint4 kx = ks[(long long)src * src_stride + c];
    const uint4 vx = vs[(long long)src * src_stride + c];
    kd[(long long)dst * CPR + c] = kx;
    vd[(long long)dst * CPR + c] = vx;
    if (km && src >= closed_rows) {
      km[(long long)(src - closed_rows) * CPR + c] = kx;
      vm[(long long)(src - closed_rows) * CPR + c] = vx;
    }
  }
}

__global__ void cache_commit_seq_meta(const Problem p, unsigned char *cache, const CacheGeom g, const int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= p.B * p.Hkv) return;
  const int b = i / p.Hkv, h = i % p.Hkv;
  int *meta = meta_of(cache, g, p, b, h);
  const int n_full = n / p.S;
  if (n_full > 0) {
    if (p.policy[h] & SEGATTN_PAST) meta[META_POOL] += n_full * p.S;
    meta[META_TAIL] = p.T;
    meta[META_RET] = 0;
  }
  meta[META_FILL] = n % p.S;
}

// One new row k,v [B,Hkv,D] per sequence -> open segment; fill += 1.  One wave per (b,h).
template <int D>
__global__ __launch_bounds__(64) void cache_decode_append_kernel(const Problem p, const CopyArgs a) {
  constexpr int CPR = D / 8;
  const int b = blockIdx.x / p.Hkv, h = blockIdx.x % p.Hkv;
  int *meta = meta_of(a.cache, a.geom, p, b, h);
  const int fill = meta[META_FILL];
  const int row = ((p.policy[h] & SEGATTN_PAST) ? meta[META_POOL] : p.T) + fill;
  __syncthreads();
  const int t = threadIdx.x;
  if (t < 2 * CPR) {
    const bool is_v = t >= CPR;
    const int c = is_v ? t - CPR : t;
    const uint4 *src = (const uint4 *)((is_v ? a.v : a.k) + ((long long)b * p.Hkv + h) * D);
    uint4 *dst = (uint4 *)(a.cache + (is_v ? v_block_off(p, a.geom, b, h) : k_block_off(p, a.geom, b, h)));
    const uint4 x = src[c];
    dst[(long long)row * CPR + c] = x;
    if (uses_view(p, a.geom, h)) {
      uint4 *mir = (uint4 *)(a.cache + (is_v ? view_v_off(p, a.geom, b, h) : view_k_off(p, a.geom, b, h)));
      mir[(long long)(a.geom.ret_cap + fill) * CPR + c] = x;
    }
  }
  if (t == 0) meta[META_FILL] = fill + 1;
}

// Explicit rows k,v [B,rows,D] -> pool of one PAST head.  grid = (row chunks, B).  The pool
// counter is advanced by cache_pool_add_kernel afterwards.
template <int D>
__global__ __launch_bounds__(256) void cache_past_append_kernel(const Problem p, const CopyArgs a) {
  constexpr int CPR = D / 8;
  const int b = blockIdx.y, h = a.kv_head;
  const int pool = meta_of(a.cache, a.geom, p, b, h)[META_POOL];
  const uint4 *ks = (const uint4 *)(a.k + (long long)b * a.m * D);
  const uint4 *vs = (const uint4 *)(a.v + (long long)b * a.m * D);
  uint4 *kd = (uint4 *)(a.cache + k_block_off(p, a.geom, b, h)) + (long long)pool * CPR;
  uint4 *vd = (uint4 *)(a.cache + v_block_off(p, a.geom, b, h)) + (long long)pool * CPR;
  const long long n = (long long)a.m * CPR;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
    kd[i] = ks[i];
    vd[i] = vs[i];
  }
}

__global__ void cache_pool_add_kernel(const Problem p, unsigned char *cache, const CacheGeom g,
                                      const int h, const int rows) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < p.B) meta_of(cache, g, p, b, h)[META_POOL] += rows;
}

// Hide the n oldest pool rows of one PAST head; rows of the current tail window stay visible
// when the head also has the TAIL bit.
// keep < 0: hide n more rows; keep >= 0: hide as many as leave at most `keep` rows visible.
__global__ void cache_evict_kernel(const Problem p, unsigned char *cache, const CacheGeom g, const int h,
                                   long long n, const long long keep) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= p.B) return;
  int *meta = meta_of(cache, g, p, b, h);
  const long long lo = meta[META_LO];
  long long limit = meta[META_POOL];
  if (keep >= 0) n = limit - lo > keep ? limit - lo - keep : 0;
  if (p.policy[h] & SEGATTN_TAIL) limit -= meta[META_TAIL];
  // at most the rows still visible below the limit (n may be anything up to INT64_MAX)
  const long long room = limit > lo ? limit - lo : 0;
  meta[META_LO] = (int)(lo + (n < room ? n : room));
}

// Counters of a chunk of sequences as the caller declares them (seg_kv_set_lengths): pool rows
// of a PAST head = the rows in closed segments, nothing evicted, no retrieved prefix.
__global__ void cache_set_lengths_kernel(const Problem p, unsigned char *cache, const CacheGeom g,
                                         const LengthsArgs a) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.count * p.Hkv) return;
  const int s = i / p.Hkv, h = i % p.Hkv;
  int *meta = meta_of(cache, g, p, a.b0 + s, h);
  meta[META_POOL] = (p.policy[h] & SEGATTN_PAST) ? a.closed[s] : 0;
  meta[META_TAIL] = a.tail[s];
  meta[META_FILL] = a.fill[s];
  meta[META_LO] = 0;
  meta[META_RET] = 0;
  meta[5] = meta[6] = meta[7] = 0;
}

// Retrieved prefix of every PAST head (Appendix D "Output"): pool rows idx[b][past head][0..R)
// -> rows [ret_cap - R, ret_cap) of the head's attention view, in list order.  An index is
// clamped into the pool, so a bad list cannot read outside the arena.  grid = (row chunks,
// B * n_past); the first block of each (b, head) also records R.
template <int D>
__global__ __launch_bounds__(256) void cache_select_kernel(const Problem p, const SelectArgs a) {
  constexpr int CPR = D / 8;
  const int b = blockIdx.y / p.n_past, np = blockIdx.y % p.n_past;
  const int h = p.order[np];  // PAST heads come first in `order`, by ascending head index
  int *meta = meta_of(a.cache, a.geom, p, b, h);
  const int pool = meta[META_POOL];
  const int *idx = a.idx + ((long long)b * p.n_past + np) * a.R;
  const uint4 *ks = (const uint4 *)(a.cache + k_block_off(p, a.geom, b, h));
  const uint4 *vs = (const uint4 *)(a.cache + v_block_off(p, a.geom, b, h));
  uint4 *kd = (uint4 *)(a.cache + view_k_off(p, a.geom, b, h)) + (long long)(a.geom.ret_cap - a.R) * CPR;
  uint4 *vd = (uint4 *)(a.cache + view_v_off(p, a.geom, b, h)) + (long long)(a.geom.ret_cap - a.R) * CPR;
  const int c = threadIdx.x % CPR;
  for (int r = blockIdx.x * (256 / CPR) + threadIdx.x / CPR; r < a.R; r += gridDim.x * (256 / CPR)) {
    int j = idx[r];
    j = j < 0 ? 0 : (j >= pool ? pool - 1 : j);
    if (pool > 0) {
      vd[(long long)r * CPR + c] = vs[(long long)j * CPR + c];
      if (!a.rope) {
        kd[(long long)r * CPR + c] = ks[(long long)j * CPR + c];
      } else if (c < CPR / 2) {
        // RoPE re-indexing of a retrieved prefix (Appendix E): the pool holds K rotated by the
        // token's absolute position j; list entry r moves to position pool - R + r, i.e. the R
        // rows become the R tokens just before the segment that starts at position `pool`.
        uint4 lo = ks[(long long)j * CPR + c], hi = ks[(long long)j * CPR + c + CPR / 2];
        rerotate8(lo, hi, (double)(pool - a.R + r - j), a.inv_freq, 8 * c);
        kd[(long long)r * CPR + c] = lo;
        kd[(long long)r * CPR + c + CPR / 2] = hi;
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) meta[META_RET] = pool > 0 ? a.R : 0;
}

// Retrieved prefixes of a whole prompt (stateless retrieval mode; Appendix D "Output"): rows
// idx[b][segment][PAST head][0..R) of the token-major k / v -> R dense rows per (b, segment, head),
// in list order.  An index is clamped into the segment's history [0, segment start), so a bad list
// cannot read outside the prompt.  With RoPE the pool rows carry their absolute positions and list
// entry r moves to position s - R + r, s the segment start (Appendix E up to a common shift).
// grid = (row chunks, B * n_seg * n_past).
template <int D>
__global__ __launch_bounds__(256) void gather_seq_kernel(const Problem p, const GatherSeqArgs a) {
  constexpr int CPR = D / 8;
  const int np = blockIdx.y % p.n_past;
  const int seg = (blockIdx.y / p.n_past) % a.n_seg;
  const int b = blockIdx.y / (p.n_past * a.n_seg);
  if (seg == 0) return;  // no history: no prefix
  const int h = p.order[np];
  const int pool = seg * p.S;
  const long long slot = ((long long)b * a.n_seg + seg) * p.n_past + np;
  const int *idx = a.idx + slot * a.R;
  const long long kv_stride = (long long)p.Hkv * CPR;  // uint4 per token row
  const uint4 *ks = (const uint4 *)a.k + ((long long)b * a.n * p.Hkv + h) * CPR;
  const uint4 *vs = (const uint4 *)a.v + ((long long)b * a.n * p.Hkv + h) * CPR;
  uint4 *kd = (uint4 *)a.ret_k + slot * a.R * CPR;
  uint4 *vd = (uint4 *)a.ret_v + slot * a.R * CPR;
  const int c = threadIdx.x % CPR;
  for (int r = blockIdx.x * (256 / CPR) + threadIdx.x / CPR; r < a.R; r += gridDim.x * (256 / CPR)) {
    int j = idx[r];
    j = j < 0 ? 0 : (j >= pool ? pool - 1 : j);
    vd[(long long)r * CPR + c] = vs[(long long)j * kv_stride + c];
    if (!a.rope) {
      kd[(long long)r * CPR + c] = ks[(long long)j * kv_stride + c];
    } else if (c < CPR / 2) {
      uint4 lo = ks[(long long)j * kv_stride + c], hi = ks[(long long)j * kv_stride + c + CPR / 2];
      rerotate8(lo, hi, (double)(pool - a.R + r - j), a.inv_freq, 8 * c);
      kd[(long long)r * CPR + c] = lo;
      kd[(long long)r * CPR + c + CPR / 2] = hi;
    }
  }
}

// ---- launchers ----------------------------------------------------------------------------
hipError_t launch_gather_seq(const Problem &p, const GatherSeqArgs &a, hipStream_t st) {
  const int rows_per_block = 256 / (p.D / 8);
  int chunks = (a.R + rows_per_block - 1) / rows_per_block;
  if (chunks < 1) chunks = 1;
  const dim3 grid(chunks, p.B * a.n_seg * p.n_past);
  if (p.D == 128) hipLaunchKernelGGL(gather_seq_kernel<128>, grid, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(gather_seq_kernel<64>, grid, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_cache_reset(const Problem &p, unsigned char *cache, const CacheGeom &g, hipStream_t st) {
  const int n = p.B * p.Hkv * kMetaInts;
  hipLaunchKernelGGL(cache_reset_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, cache, g);
  return hipGetLastError();
}

hipError_t launch_cache_append(const Problem &p, const CopyArgs &a, hipStream_t st) {
  const int cpr = p.D / 8;
  const int rows_per_block = 256 / cpr * 8;
  const dim3 grid((a.m + rows_per_block - 1) / rows_per_block, p.B * p.Hkv);
  if (p.D == 128) hipLaunchKernelGGL(cache_append_kernel<128>, grid, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(cache_append_kernel<64>, grid, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_cache_commit_seq(const Problem &p, const CopyArgs &a, hipStream_t st) {
  const int cpr = p.D / 8, rows_per_block = 256 / cpr * 8;
  const int n = a.m, open = n % p.S;
  int max_rows = p.T + open;  // rows written for a non-PAST head
  if (p.n_past > 0 && n > max_rows) max_rows = n;
  if (max_rows > 0) {
    const dim3 grid((unsigned)((max_rows + rows_per_block - 1) / rows_per_block), (unsigned)(p.B * p.Hkv));
    if (p.D == 128) hipLaunchKernelGGL(cache_commit_seq_kernel<128>, grid, dim3(256), 0, st, p, a);
    else hipLaunchKernelGGL(cache_commit_seq_kernel<64>, grid, dim3(256), 0, st, p, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(cache_commit_seq_meta, dim3((p.B * p.Hkv + 63) / 64), dim3(64), 0, st, p, a.cache, a.geom, n);
  return hipGetLastError();
}

hipError_t launch_cache_close(const Problem &p, unsigned char *cache, const CacheGeom &g, int add,
                              hipStream_t st) {
  const dim3 grid(p.B * p.Hkv);
  if (p.D == 128) hipLaunchKernelGGL(cache_close_kernel<128>, grid, dim3(256), 0, st, p, cache, g, add);
  else hipLaunchKernelGGL(cache_close_kernel<64>, grid, dim3(256), 0, st, p, cache, g, add);
  return hipGetLastError();
}

hipError_t launch_cache_decode_append(const Problem &p, const CopyArgs &a, hipStream_t st) {
  const dim3 grid(p.B * p.Hkv);
  if (p.D == 128) hipLaunchKernelGGL(cache_decode_append_kernel<128>, grid, dim3(64), 0, st, p, a);
  else hipLaunchKernelGGL(cache_decode_append_kernel<64>, grid, dim3(64), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_cache_past_append(const Problem &p, const CopyArgs &a, hipStream_t st) {
  const long long n = (long long)a.m * (p.D / 8);
  long long blocks = (n + 2047) / 2048;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  const dim3 grid((unsigned)blocks, p.B);
  if (p.D == 128) hipLaunchKernelGGL(cache_past_append_kernel<128>, grid, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(cache_past_append_kernel<64>, grid, dim3(256), 0, st, p, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cache_pool_add_kernel, dim3((p.B + 63) / 64), dim3(64), 0, st, p, a.cache, a.geom,
                     a.kv_head, a.m);
  return hipGetLastError();
}

hipError_t launch_cache_select(const Problem &p, const SelectArgs &a, hipStream_t st) {
  const int rows_per_block = 256 / (p.D / 8);
  int chunks = (a.R + rows_per_block - 1) / rows_per_block;
  if (chunks < 1) chunks = 1;
  const dim3 grid(chunks, p.B * p.n_past);
  if (p.D == 128) hipLaunchKernelGGL(cache_select_kernel<128>, grid, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(cache_select_kernel<64>, grid, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_cache_set_lengths(const Problem &p, unsigned char *cache, const CacheGeom &g, const LengthsArgs &a,
                                    hipStream_t st) {
  const int n = a.count * p.Hkv;
  hipLaunchKernelGGL(cache_set_lengths_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, cache, g, a);
  return hipGetLastError();
}

hipError_t launch_cache_evict(const Problem &p, unsigned char *cache, const CacheGeom &g, int kv_head,
                              long long n_oldest, long long keep, hipStream_t st) {
  hipLaunchKernelGGL(cache_evict_kernel, dim3((p.B + 63) / 64), dim3(64), 0, st, p, cache, g, kv_head,
                     n_oldest, keep);
  return hipGetLastError();
}

}  // namespace segattn
