// Work decomposition shared by the prefill kernels of libsegattn: which workgroup handles
// which (sequence, KV head, head sub-group, segment, query block), and where its keys live.
//
// A workgroup's keys form two spans: span 0 = the prefix the head's policy grants (carried
// tail and/or past rows -- the whole pool or, in retrieval mode, the gathered rows of the
// head's attention view -- Eq. 13; every row visible to every query of the workgroup) and
// span 1 = the rows of the query's own segment (causal, Eq. 12's mask).
#pragma once
#include "segattn_internal.h"

namespace segattn {

// One workgroup's share of the problem.
struct WorkItem {
  const unsigned short *k0, *v0, *k1, *v1;  // first row of span 0 / span 1 for this KV head
  long long stride0, stride1;               // elements between consecutive rows
  int n0, n1;                               // rows in span 0; rows of the segment present
  const unsigned short *q;                  // row 0 of the segment's queries, head 0
  unsigned char *out;                       // row 0 of the segment's outputs, head 0
  float *lse;                               // lse of (b, head 0, segment row 0)
  long long lse_head_stride;                // floats between heads in lse
  int t0;                                   // first in-segment query row of the workgroup
  int kv, hsub, b;
  // Where the MFMA prefill kernel writes: rows of `out_heads` heads, this workgroup's first head
  // at `ohead0`, fp32 if `wide`.  Normally the caller's tensor; the workspace for a split prefix.
  int nq;                                   // query rows of the segment present (n1, except for a prefix piece)
  int out_heads, ohead0;
  bool wide;
  bool valid;
};

// ---- work items from queues (kernels that run as a resident grid)
// Queue y (counter at queue[kQueueStride * y]) holds the items y, y+8, ... of a launch of
// `n_items`, in order: what XCD y would be dealt if every item were a workgroup of its own.  A
// workgroup (on XCD blockIdx.x % 8) takes from its XCD's queue first; once that is empty, from the
// queue with the most items left (the XCD furthest behind); -1 when all are empty.  Thread 0 does
// the work, `slot` (shared memory) carries the answer to the others; two workgroup barriers.
// drawn / ticket: thread 0 may already hold a position drawn from the own queue (by atomicAdd,
// while the previous item was finishing), so that the round trip is over by now.
__device__ __forceinline__ int take_item(unsigned *queue, int n_items, bool drawn, unsigned ticket, int *slot) {
  if (threadIdx.x == 0) {
    auto items_of = [&](int y) { return y < n_items ? (unsigned)(n_items - y + 7) >> 3 : 0u; };
    const int x = (int)blockIdx.x & 7;
    int got = -1;
    const unsigned j0 = drawn ? ticket : atomicAdd(queue + kQueueStride * x, 1u);
    if (j0 < items_of(x)) {
      got = 8 * (int)j0 + x;
    } else {
      // Counters only grow, so a queue seen empty stays empty; a failed attempt marks its queue
      // empty: at most eight attempts.
      unsigned left[8];
#pragma unroll
      for (int y = 0; y < 8; ++y) {
        const unsigned at = __hip_atomic_load(queue + kQueueStride * y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        left[y] = at < items_of(y) ? items_of(y) - at : 0u;
      }
#pragma unroll 1
      for (int t = 0; t < 8 && got < 0; ++t) {
        unsigned most = 0;
        int y = -1;
#pragma unroll
        for (int z = 0; z < 8; ++z)
          if (left[z] > most) {
            most = left[z];
            y = z;
          }
        if (y < 0) break;
        const unsigned j = atomicAdd(queue + kQueueStride * y, 1u);
        if (j < items_of(y)) got = 8 * (int)j + y;
#pragma unroll
        for (int z = 0; z < 8; ++z)
          if (z == y) left[z] = 0;
      }
    }
    *slot = got;
  }
  __syncthreads();
  const int bid = __builtin_amdgcn_readfirstlane(*slot);
  __syncthreads();  // everyone has read it before thread 0 writes the next one
  return bid;
}

// Item index -> (segment, query block, head list position, sequence, head sub-group, prefix piece):
// all PAST items by descending absolute query block (longest work first), then the others grouped
// so that the query blocks sharing K/V rows run together on one XCD.  Pure integer arithmetic, the
// same on the host (where it is tested for being a one-to-one map) and on the device.
// total_items: items of the launch (PrefillArgs::grid_items, or the grid size).
struct ItemCoords {
  int seg, qblk, hidx, b, hs, part;
};
__host__ __device__ inline ItemCoords item_coords(const Problem &p, const PrefillArgs &a, int bid, int total_items,
                                                  int heads_per_wg) {
  const int nhs = p.g / heads_per_wg;
  const int nqb = a.q_blocks_per_seg;
  // heads listed first, longest work first: the PAST heads -- unless they attend to a retrieved
  // prefix of bounded size, in which case their key ranges are as short as everybody's and all
  // heads go into the common list below
  const int n_first = ((a.cache != nullptr && a.geom.ret_cap > 0) || a.ret_k != nullptr) ? 0 : p.n_past;
  const int n_other = p.Hkv - n_first;
  const int parts = (a.cache != nullptr && a.parts > 1) ? a.parts : 1;
  const long long past_items = (long long)p.B * n_first * nhs * a.n_seg * nqb * parts;
  int seg, qblk, hidx, b, hs, part = 0;
  if (a.dv.ok) {
    // the same arithmetic as the branches below with the launch's divisors prepared by the host
    // (every quantity is below 2^31 then): a few scalar multiplies instead of a dozen divisions
    const ResolveDivs &dv = a.dv;
    if (bid < past_items) {
      const int row = fast_div(bid, dv.per);
      const int gq = a.n_seg * nqb - 1 - row;
      int rest = bid - row * (int)dv.per.d;
      if (a.cu_seqlens) rest = fast_mod(rest + row, dv.per);
      part = fast_mod(rest, dv.parts);
      rest = fast_div(rest, dv.parts);
      seg = fast_div(gq, dv.nqb);
      qblk = gq - seg * nqb;
      hs = fast_mod(rest, dv.nhs);
      rest = fast_div(rest, dv.nhs);
      b = fast_div(rest, dv.n_first);
      hidx = rest - b * (int)dv.n_first.d;
    } else {
      const int pi = (int)past_items;
      const int items = total_items - pi;
      const int x = bid & 7;
      int start = 0, first = 0;
#pragma unroll
      for (int xx = 0; xx < 8; ++xx) {
        const int o = (xx - pi) & 7;
        const int cnt = o < items ? (items - o + 7) >> 3 : 0;
        if (xx < x) start += cnt;
        if (xx == x) first = pi + o;
      }
      const int L = start + ((bid - first) >> 3);
      const int d = (int)dv.sub.d;
      const int sg = fast_div(L, dv.per_sub);
      const int grp = fast_div(sg, dv.sub);
      qblk = nqb - 1 - ((sg - grp * d) + d * (L - sg * (int)dv.per_sub.d));
      const long long shuffled = (long long)grp * (a.pair_stride > 0 ? a.pair_stride : 1);  // < 2^31 (host check)
      int rest = fast_mod((int)shuffled, dv.groups);
      hs = fast_mod(rest, dv.nhs);
      rest = fast_div(rest, dv.nhs);
      const int r2 = fast_div(rest, dv.n_other);
      hidx = n_first + (rest - r2 * (int)dv.n_other.d);
      seg = fast_div(r2, dv.batch);
      b = r2 - seg * (int)dv.batch.d;
    }
  } else if (bid < past_items) {
    const int per = p.B * n_first * nhs * parts;
    const int gq = a.n_seg * nqb - 1 - bid / per;
    int rest = bid % per;
    // Packed batch of unequal sequences: the workgroups of one query block index are `per` in a
    // row, and where `per` is a multiple of 8 a given (sequence, head) would meet the same XCD at
    // every index -- the long sequences' XCDs would work on while the others idle.  Rotate.
    if (a.cu_seqlens) rest = (rest + bid / per) % per;
    part = rest % parts;
    rest /= parts;
    seg = gq / nqb;
    qblk = gq % nqb;
    hs = rest % nhs;
    rest /= nhs;
    hidx = rest % n_first;
    b = rest / n_first;
  } else {
    // Heads without the PAST bit: the query blocks of one (sequence, head, segment) read the same
    // few MB of K/V, so they should run at the same time behind the same L2.  Workgroups go to the
    // 8 XCDs (one L2 each) round-robin by index: XCD x = bid % 8 takes the bids x, x+8, ... in
    // order.  Give each XCD a contiguous range of the list ordered by (segment, sequence, head,
    // head sub-group) and, inside one of those, by descending query block.
    const long long items = (long long)total_items - past_items;
    const int x = bid & 7;
    long long start = 0, first = 0;
#pragma unroll
    for (int xx = 0; xx < 8; ++xx) {
      const long long o = (xx - past_items) & 7;  // first list position served by XCD xx
      const long long cnt = o < items ? (items - o + 7) >> 3 : 0;
      if (xx < x) start += cnt;
      if (xx == x) first = past_items + o;
    }
    long long L = start + ((bid - first) >> 3);
    // Position L of the list -> (group, query block).  Every XCD takes its workgroups in index
    // order, so at equal speed the XCDs advance in step and the j-th blocks of all XCDs should
    // be equally long: that holds
    // if every XCD's range is a whole number of groups.  Where the group count is no multiple of 8
    // the launcher deals each group's blocks into d interleaved sub-groups (block q belongs to
    // sub-group (nqb-1-q) % d), each with the group's length profile, and the list runs over those.
    const int d = a.sub_groups > 1 ? a.sub_groups : 1;
    const int per_sub = nqb / d;
    const long long sg = L / per_sub;
    qblk = nqb - 1 - ((int)(sg % d) + d * (int)(L % per_sub));
    L = (sg / d) * nqb;  // first position of the group, for the group index below
    // Consecutive groups differ little in length for a dense batch but a lot for a ragged one (a
    // whole range of them can be empty): a multiplicative shuffle of the group index (stride
    // coprime to the group count, about an eighth of it) deals each XCD an even sample.
    const long long groups = items / nqb;
    int rest = (int)((L / nqb) * (a.pair_stride > 0 ? a.pair_stride : 1) % groups);
    hs = rest % nhs;
    rest /= nhs;
    hidx = n_first + rest % n_other;
    rest /= n_other;
    b = rest % p.B;
    seg = rest / p.B;
  }
  return ItemCoords{seg, qblk, hidx, b, hs, part};
}

// blockIdx -> work item: the coordinates above, then the item's key spans, query rows and outputs.
__device__ inline WorkItem resolve(const Problem &p, const PrefillArgs &a, int bid, int rows_per_wg,
                                   int heads_per_wg) {
  WorkItem w;
  const int parts = (a.cache != nullptr && a.parts > 1) ? a.parts : 1;
  const ItemCoords ic = item_coords(p, a, bid, a.grid_items > 0 ? a.grid_items : (int)gridDim.x, heads_per_wg);
  const int seg = ic.seg, qblk = ic.qblk, hidx = ic.hidx, b = ic.b, hs = ic.hs, part = ic.part;
  const int kv = p.order[hidx];
  const int pol = p.policy[kv];
  w.kv = kv;
  w.hsub = hs;
  w.b = b;
  w.t0 = qblk * rows_per_wg;
  const long long kv_stride = (long long)p.Hkv * p.D;
  if (a.cache == nullptr) {  // SEQ mode: prefix read from k/v by absolute position
    // dense batch: sequence b occupies rows [b*N, (b+1)*N); packed ragged batch: rows
    // [cu[b], cu[b+1]) and lse is [Hq, total rows]
    long long N = a.n_rows, base = (long long)b * N, lse_base = (long long)b * p.Hq * N, lse_stride = N;
    if (a.cu_seqlens) {
      base = a.cu_seqlens[b];
      N = a.cu_seqlens[b + 1] - base;
      lse_base = base;
      lse_stride = a.total_rows;
    }
    const long long s = (long long)seg * p.S;
    const long long m_i = (N - s < p.S) ? (N - s) : p.S;  // <= 0 beyond the end of a short sequence
    long long lo = s;
    if (pol & SEGATTN_PAST) lo = 0;
    else if (pol & SEGATTN_TAIL) lo = (s - p.T > 0) ? s - p.T : 0;
    w.n0 = (int)(s - lo);
    w.n1 = (int)m_i;
    w.k0 = a.k + (base + lo) * kv_stride + (long long)kv * p.D;
    w.v0 = a.v + (base + lo) * kv_stride + (long long)kv * p.D;
    w.k1 = a.k + (base + s) * kv_stride + (long long)kv * p.D;
    w.v1 = a.v + (base + s) * kv_stride + (long long)kv * p.D;
    w.stride0 = w.stride1 = kv_stride;
    if (a.ret_k != nullptr && (pol & SEGATTN_PAST)) {
      // retrieved prefix of (b, segment, head): R dense gathered rows (none for the first segment)
      const long long slot = ((long long)b * a.n_seg + seg) * p.n_past + p.past_before[kv];
      w.n0 = seg > 0 ? a.ret_R : 0;
      w.k0 = a.ret_k + slot * a.ret_R * p.D;
      w.v0 = a.ret_v + slot * a.ret_R * p.D;
      w.stride0 = p.D;
    }
    w.q = a.q + (base + s) * p.Hq * p.D;
    const long long osz = p.out_fp32 ? 4 : 2;
    w.out = (unsigned char *)a.out + (base + s) * p.Hq * p.D * osz;
    w.lse = a.lse + lse_base + s;
    w.lse_head_stride = lse_stride;
  } else {  // CTX mode: prefix (and the committed part of the open segment) from the cache
    const int *meta = (const int *)(a.cache + a.geom.meta_off) + ((long long)b * p.Hkv + kv) * kMetaInts;
    int lo, seg_row0;
    window_of(p, a.geom, kv, meta, lo, seg_row0);
    const int hi = seg_row0 + meta[META_FILL];
    const long long m = a.n_rows;
    w.n0 = hi - lo;
    w.n1 = (int)m;
    w.k0 = (const unsigned short *)(a.cache + attn_k_off(p, a.geom, b, kv)) + (long long)lo * p.D;
    w.v0 = (const unsigned short *)(a.cache + attn_v_off(p, a.geom, b, kv)) + (long long)lo * p.D;
    w.stride0 = p.D;
    w.k1 = a.k + (long long)b * m * kv_stride + (long long)kv * p.D;
    w.v1 = a.v + (long long)b * m * kv_stride + (long long)kv * p.D;
    w.stride1 = kv_stride;
    w.q = a.q + (long long)b * m * p.Hq * p.D;
    const long long osz = p.out_fp32 ? 4 : 2;
    w.out = (unsigned char *)a.out + (long long)b * m * p.Hq * p.D * osz;
    w.lse = a.lse + (long long)b * p.Hq * m;
    w.lse_head_stride = m;
  }
  w.nq = w.n1;
  w.out_heads = p.Hq;
  w.ohead0 = kv * p.g + hs * heads_per_wg;
  w.wide = p.out_fp32 != 0;
  if (parts > 1 && (pol & SEGATTN_PAST)) {
    // Piece `part` of the prefix.  The last piece also takes the open segment (about n1/2 keys per
    // query on average), so the others get a little more of the prefix: t rows each, a multiple of
    // the 32-key step, and the last one the rest (the host only splits prefixes of >= 1024 rows per
    // piece, so the rest is never empty).
    const int n0 = w.n0;
    int t = ((n0 + w.n1 / 2) / parts + 31) & ~31;
    const int t_max = ((n0 - 32) / (parts - 1)) & ~31;
    t = t < t_max ? t : t_max;
    const int start = part * t;
    w.k0 += (long long)start * p.D;
    w.v0 += (long long)start * p.D;
    w.n0 = (part == parts - 1) ? n0 - start : t;
    if (part != parts - 1) w.n1 = 0;
    const int ph = p.n_past * p.g;  // heads per workspace row
    const long long m = a.n_rows;
    w.out = (unsigned char *)(a.part_out + (((long long)b * parts + part) * m * ph) * p.D);
    w.lse = a.part_lse + ((long long)b * parts + part) * ph * m;
    w.lse_head_stride = m;
    w.out_heads = ph;
    w.ohead0 = p.past_before[kv] * p.g + hs * heads_per_wg;
    w.wide = true;
  }
  w.valid = w.t0 < w.nq;
  return w;
}

__device__ inline int uniform_i32(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ inline long long uniform_i64(long long x) {
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(unsigned long long)x);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)x >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}
template <typename T>
__device__ inline T *uniform_ptr(T *ptr) {
  const unsigned long long u = (unsigned long long)ptr;
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)u);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(u >> 32));
  return (T *)(((unsigned long long)hi << 32) | lo);
}
// Everything in a work item is the same for the whole workgroup, but some of it comes from memory
// (sequence offsets, cache counters) through vector loads.  Pin the sizes and the K/V pointers to
// scalar registers so that loader pointers and loop bounds derived from them stay out of the
// vector file.
__device__ inline void pin_uniform(WorkItem &w) {
  w.n0 = uniform_i32(w.n0);
  w.n1 = uniform_i32(w.n1);
  w.nq = uniform_i32(w.nq);
  w.t0 = uniform_i32(w.t0);
  w.stride0 = uniform_i32((int)w.stride0);
  w.stride1 = uniform_i32((int)w.stride1);
  w.k0 = uniform_ptr(w.k0);
  w.v0 = uniform_ptr(w.v0);
  w.k1 = uniform_ptr(w.k1);
  w.v1 = uniform_ptr(w.v1);
}

__device__ inline float bf16_bits_to_f32(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

}  // namespace segattn
